"""ctypes front end of the CPU oracle (``sq_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg do.
Every function marshals numpy arrays into the C routine of the same name; the
arithmetic lives in the C file, which cites the passages of the paper it
follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sq_oracle.c")
_LIB = os.path.join(_HERE, "libsq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 scalar loops, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-D_GNU_SOURCE",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        lib.sqo_half_to_double.restype = C.c_double
        lib.sqo_half_to_double.argtypes = [C.c_uint16]
        lib.sqo_double_to_half.restype = C.c_uint16
        lib.sqo_double_to_half.argtypes = [C.c_double]
        lib.sqo_art_angle.restype = C.c_double
        lib.sqo_art_angle.argtypes = [C.c_double, C.c_double]
        lib.sqo_givens_apply.restype = None
        lib.sqo_givens_apply.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_double]
        lib.sqo_kron_apply.restype = None
        lib.sqo_kron_apply.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                       C.c_void_p, C.c_void_p]
        lib.sqo_kron_apply_dense.restype = None
        lib.sqo_kron_apply_dense.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                             C.c_void_p]
        lib.sqo_rotate.restype = C.c_int
        lib.sqo_rotate.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int64,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                   C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
        lib.sqo_quantize_rows.restype = C.c_int
        lib.sqo_quantize_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]
        lib.sqo_quantize_rows_f32.restype = C.c_int
        lib.sqo_quantize_rows_f32.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]
        lib.sqo_quantize_rows_variant.restype = C.c_int
        lib.sqo_quantize_rows_variant.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_double,
                                                  C.c_void_p, C.c_void_p]
        lib.sqo_pack_w3.restype = C.c_int
        lib.sqo_pack_w3.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        lib.sqo_unpack_w3.restype = C.c_int
        lib.sqo_unpack_w3.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        lib.sqo_tile_weights_decode.restype = C.c_int
        lib.sqo_tile_weights_decode.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_int]
        lib.sqo_unpack_codes.restype = None
        lib.sqo_unpack_codes.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        lib.sqo_gemm.restype = C.c_int
        lib.sqo_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int,
                                 C.c_void_p, C.c_void_p, C.c_int,
                                 C.c_void_p, C.c_int64, C.c_void_p]
        lib.sqo_gemm_acc_at.restype = C.c_int64
        lib.sqo_gemm_acc_at.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64]
        lib.sqo_round_rows_to_half.restype = None
        lib.sqo_round_rows_to_half.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_int64]
        lib.sqo_gemm_w4a16.restype = C.c_int
        lib.sqo_gemm_w4a16.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int64, C.c_void_p, C.c_void_p, C.c_int,
                                       C.c_void_p, C.c_int64, C.c_void_p]
        lib.sqo_kron_factor.restype = None
        lib.sqo_kron_factor.argtypes = [C.c_int64, C.c_void_p, C.c_void_p]
        lib.sqo_num_threads.restype = C.c_int
        lib.sqo_num_threads.argtypes = []
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


# ------------------------------------------------------------------ fp16 ---

def half_to_double(bits: int) -> float:
    return _load().sqo_half_to_double(int(bits))


def double_to_half(x: float) -> int:
    return _load().sqo_double_to_half(float(x))


# ------------------------------------------------------- Sec. 4.1, Lemma 1 ---

def art_angle(a: float, b: float) -> float:
    return _load().sqo_art_angle(float(a), float(b))


def givens_apply(row, i: int, j: int, theta: float) -> np.ndarray:
    """Return row * G(i, j; theta) for one fp64 row vector."""
    out = _c(row, np.float64).copy()
    if not (0 <= i < out.size and 0 <= j < out.size and i != j):
        raise ValueError("bad Givens pair")
    _load().sqo_givens_apply(_ptr(out), i, j, float(theta))
    return out


# ------------------------------------------------------------------ Eq. 18 ---

def kron_apply(row, R1, R2) -> np.ndarray:
    R1 = _c(R1, np.float64)
    R2 = _c(R2, np.float64)
    n1, n2 = R1.shape[0], R2.shape[0]
    row = _c(row, np.float64)
    assert R1.shape == (n1, n1) and R2.shape == (n2, n2) and row.shape == (n1 * n2,)
    out = np.empty(n1 * n2, np.float64)
    tmp = np.empty(n1 * n2, np.float64)
    _load().sqo_kron_apply(_ptr(row), _ptr(R1), n1, _ptr(R2), n2, _ptr(out), _ptr(tmp))
    return out


def kron_apply_dense(row, R1, R2) -> np.ndarray:
    R1 = _c(R1, np.float64)
    R2 = _c(R2, np.float64)
    n1, n2 = R1.shape[0], R2.shape[0]
    row = _c(row, np.float64)
    assert row.shape == (n1 * n2,)
    out = np.empty(n1 * n2, np.float64)
    _load().sqo_kron_apply_dense(_ptr(row), _ptr(R1), n1, _ptr(R2), n2, _ptr(out))
    return out


# ---------------------------------------------------------------- Sec. 4.2 ---

def rotate(X_f16, giv_i, giv_j, giv_theta, R1, R2) -> np.ndarray:
    """X: [T, K] float16.  R1, R2: any float dtype, used as fp64.  -> [T, K] fp64."""
    X = np.ascontiguousarray(X_f16)
    assert X.dtype == np.float16 and X.ndim == 2
    T, K = X.shape
    R1 = _c(R1, np.float64)
    R2 = _c(R2, np.float64)
    gi = _c(giv_i, np.int32)
    gj = _c(giv_j, np.int32)
    gt = _c(giv_theta, np.float64)
    P = gi.size
    assert gj.size == P and gt.size == P
    out = np.empty((T, K), np.float64)
    rc = _load().sqo_rotate(_ptr(X.view(np.uint16)), T, K, K, _ptr(gi), _ptr(gj), _ptr(gt), P,
                            _ptr(R1), R1.shape[0], _ptr(R2), R2.shape[0], _ptr(out))
    if rc != 0:
        raise ValueError("sqo_rotate: bad argument")
    return out


# ---------------------------------------------------------------- Sec. 3.2 ---

def quantize_rows(Xrot):
    """-> (Q uint8 [T, K/2], scales float32 [T]); decision precision follows the input dtype
    (float64 -> fp64 decisions, float32 -> fp32 decisions)."""
    Xrot = np.ascontiguousarray(Xrot)
    assert Xrot.ndim == 2 and Xrot.dtype in (np.float64, np.float32)
    T, K = Xrot.shape
    Q = np.empty((T, K // 2), np.uint8)
    s = np.empty(T, np.float32)
    fn = _load().sqo_quantize_rows if Xrot.dtype == np.float64 else _load().sqo_quantize_rows_f32
    if fn(_ptr(Xrot), T, K, _ptr(Q), _ptr(s)) != 0:
        raise ValueError("quantize_rows: bad argument")
    return Q, s


def quantize_rows_variant(Xrot, bits: int = 4, clip_ratio: float = 1.0):
    """The quantizer with ``bits`` bits (2..4) and a clipping ratio in (0, 1]: step
    ratio * max|z| / (2^(bits-1) - 1), codes clamped to [-2^(bits-1), 2^(bits-1) - 1], stored as
    nibbles.  fp64 input and decisions.  -> (Q uint8 [T, K/2], scales float32 [T])."""
    Xrot = np.ascontiguousarray(Xrot, dtype=np.float64)
    T, K = Xrot.shape
    Q = np.empty((T, K // 2), np.uint8)
    s = np.empty(T, np.float32)
    if _load().sqo_quantize_rows_variant(_ptr(Xrot), T, K, int(bits), float(clip_ratio), _ptr(Q), _ptr(s)) != 0:
        raise ValueError("quantize_rows_variant: bad argument")
    return Q, s


def pack_w3(Q) -> np.ndarray:
    """Nibble codes [N, K/2] (all in [-4, 3], K % 64 == 0) -> 3-bit storage [N, 3K/8]."""
    Q = _c(Q, np.uint8)
    N, Kh = Q.shape
    out = np.empty((N, 3 * Kh // 4), np.uint8)
    rc = _load().sqo_pack_w3(_ptr(Q), N, 2 * Kh, _ptr(out))
    if rc != 0:
        raise ValueError(f"pack_w3 failed rc={rc}")
    return out


def unpack_w3(Q3) -> np.ndarray:
    """3-bit storage [N, 3K/8] -> nibble codes [N, K/2]."""
    Q3 = _c(Q3, np.uint8)
    N, B = Q3.shape
    K = B * 8 // 3
    out = np.empty((N, K // 2), np.uint8)
    if _load().sqo_unpack_w3(_ptr(Q3), N, K, _ptr(out)) != 0:
        raise ValueError("unpack_w3: bad argument")
    return out


def tile_weights_decode(Qw) -> np.ndarray:
    """Weight codes [N, K/2] (K % 256 == 0) -> the decode layout, flat uint8 of ceil(N/32)*32*K/2 bytes."""
    Qw = _c(Qw, np.uint8)
    N, Kh = Qw.shape
    out = np.empty(((N + 31) // 32) * 32 * Kh, np.uint8)
    if _load().sqo_tile_weights_decode(_ptr(Qw), N, 2 * Kh, _ptr(out), 0) != 0:
        raise ValueError("tile_weights_decode: bad argument")
    return out


def untile_weights_decode(Qt, N: int, K: int) -> np.ndarray:
    """Inverse of tile_weights_decode."""
    Qt = _c(Qt, np.uint8)
    assert Qt.size == ((N + 31) // 32) * 32 * (K // 2)
    out = np.empty((N, K // 2), np.uint8)
    if _load().sqo_tile_weights_decode(_ptr(out), N, K, _ptr(Qt), 1) != 0:
        raise ValueError("untile_weights_decode: bad argument")
    return out


def unpack_codes(Q) -> np.ndarray:
    Q = _c(Q, np.uint8)
    T, Kh = Q.shape
    out = np.empty((T, 2 * Kh), np.int8)
    _load().sqo_unpack_codes(_ptr(Q), T, 2 * Kh, _ptr(out))
    return out


# ------------------------------------------------------------------- Eq. 1 ---

def gemm(Qx, sx, Qw, sw):
    """-> (Y float16 [T, N], acc int32 [T, N])."""
    Qx = _c(Qx, np.uint8)
    Qw = _c(Qw, np.uint8)
    sx = _c(sx, np.float32)
    sw = _c(sw, np.float32)
    T, Kh = Qx.shape
    N = Qw.shape[0]
    assert Qw.shape[1] == Kh and sx.size == T and sw.size == N
    Y = np.empty((T, N), np.uint16)
    acc = np.empty((T, N), np.int32)
    rc = _load().sqo_gemm(_ptr(Qx), _ptr(sx), T, 2 * Kh, _ptr(Qw), _ptr(sw), N, _ptr(Y), N, _ptr(acc))
    if rc != 0:
        raise ValueError(f"sqo_gemm failed rc={rc}")
    return Y.view(np.float16), acc


def gemm_acc_at(Qx, Qw, t: int, n: int) -> int:
    Qx = _c(Qx, np.uint8)
    Qw = _c(Qw, np.uint8)
    return int(_load().sqo_gemm_acc_at(_ptr(Qx), _ptr(Qw), 2 * Qx.shape[1], t, n))


def prepare_weights(Wt_f16, giv_i, giv_j, giv_theta, R1, R2):
    """Offline weight path (Sec. 4.2): rows of W^T get the same transform as token rows,
    Flat(W~_R) = W^T R, then round-to-nearest 4-bit per output channel (Table 1, 'RTN').
    Wt: [N, K] float16 (= W transposed).  -> (Qw [N, K/2], sw [N])."""
    return quantize_rows(rotate(Wt_f16, giv_i, giv_j, giv_theta, R1, R2))


# ------------------------------------------- weight-only variant (Table B.3) ---

def rotate_f16(X_f16, giv_i, giv_j, giv_theta, R1, R2) -> np.ndarray:
    """The 16-bit activations of the weight-only setting (W4A16): the rotated rows X R of
    Eq. 1, each entry rounded once from fp64 to fp16.  -> [T, K] float16."""
    xr = rotate(X_f16, giv_i, giv_j, giv_theta, R1, R2)
    T, K = xr.shape
    out = np.empty((T, K), np.uint16)
    _load().sqo_round_rows_to_half(_ptr(xr), T, K, _ptr(out), K)
    return out.view(np.float16)


def gemm_w4a16(Xh, Qw, sw, want_abs_sum=False):
    """Y = fp16(sw[n] * sum_k x[t,k] qw[n,k]) with fp16 activations and 4-bit weight codes; sums in
    fp64.  -> Y float16 [T, N] (and sw[n] * sum_k |x qw| as float64 [T, N] if asked)."""
    Xh = np.ascontiguousarray(Xh)
    assert Xh.dtype == np.float16 and Xh.ndim == 2
    Qw = _c(Qw, np.uint8)
    sw = _c(sw, np.float32)
    T, K = Xh.shape
    N = Qw.shape[0]
    assert Qw.shape[1] * 2 == K and sw.size == N
    Y = np.empty((T, N), np.uint16)
    m = np.empty((T, N), np.float64) if want_abs_sum else None
    rc = _load().sqo_gemm_w4a16(_ptr(Xh.view(np.uint16)), T, K, K, _ptr(Qw), _ptr(sw), N, _ptr(Y), N,
                                None if m is None else _ptr(m))
    if rc != 0:
        raise ValueError("sqo_gemm_w4a16: bad argument")
    return (Y.view(np.float16), m) if want_abs_sum else Y.view(np.float16)


def prepare_weights_variant(Wt_f16, giv_i, giv_j, giv_theta, R1, R2, bits=4, clip_ratio=1.0):
    """prepare_weights with the b-bit / clipped quantizer (W3A16 of the weight-only table)."""
    return quantize_rows_variant(rotate(Wt_f16, giv_i, giv_j, giv_theta, R1, R2), bits, clip_ratio)


def gemm_w3a16(Xh, Qw3, sw, want_abs_sum=False):
    """gemm_w4a16 on weights kept in the 3-bit storage."""
    return gemm_w4a16(Xh, unpack_w3(Qw3), sw, want_abs_sum)


# ------------------------------------------------------------------ Alg. 1 ---

def kron_factor(n: int):
    a = C.c_int64(0)
    b = C.c_int64(0)
    _load().sqo_kron_factor(int(n), C.byref(a), C.byref(b))
    return a.value, b.value


def num_threads() -> int:
    return _load().sqo_num_threads()
