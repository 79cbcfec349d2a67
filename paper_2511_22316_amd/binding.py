"""Thin ctypes binding of ``libsinglequant.so`` (declared in ``include/singlequant.h``).

Argument marshalling only: every step of the path runs inside the HIP library.  torch is used
for device memory and streams.  There is no fallback: if the library has not been built the
first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsinglequant.so")
_lib = None

SQ_OK = 0


class SQError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"singlequant: {text} (status {code})")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2511_22316_amd.build` "
                "(there is no CPU fallback)")
        # torch first: it brings its own copy of the HIP runtime, and the device memory this binding
        # passes around belongs to that copy.  Loaded the other way round (this library, which
        # names the runtime of the ROCm installation, before torch) the process ends up with two
        # runtimes, and the one the library talks to reports "no ROCm-capable device".
        import torch  # noqa: F401
        lib = C.CDLL(_LIB_PATH)
        lib.sq_rotate_quantize.restype = C.c_int
        lib.sq_rotate_quantize.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.sq_prepared_rotation_bytes.restype = C.c_int64
        lib.sq_prepared_rotation_bytes.argtypes = [C.c_int32, C.c_int32]
        lib.sq_prepare_rotation.restype = C.c_int
        lib.sq_prepare_rotation.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        lib.sq_rotate_quantize_prepared.restype = C.c_int
        lib.sq_rotate_quantize_prepared.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.sq_decode_layer_workspace_bytes.restype = C.c_int64
        lib.sq_decode_layer_workspace_bytes.argtypes = [C.c_int64, C.c_int32]
        lib.sq_decode_layer.restype = C.c_int
        lib.sq_decode_layer.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.sq_decode_layer_static.restype = C.c_int
        lib.sq_decode_layer_static.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
        lib.sq_rotate_fp16.restype = C.c_int
        lib.sq_rotate_fp16.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int64, C.c_void_p]
        lib.sq_w4a16_gemm.restype = C.c_int
        lib.sq_w4a16_gemm.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int64, C.c_void_p]
        lib.sq_decode_weights_bytes.restype = C.c_int64
        lib.sq_decode_weights_bytes.argtypes = [C.c_int32, C.c_int32]
        lib.sq_tile_weights_decode.restype = C.c_int
        lib.sq_tile_weights_decode.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.sq_w4a4_gemm_decode.restype = C.c_int
        lib.sq_w4a4_gemm_decode.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.sq_w3a16_gemm.restype = C.c_int
        lib.sq_w3a16_gemm.argtypes = lib.sq_w4a16_gemm.argtypes
        lib.sq_pack_w3.restype = C.c_int
        lib.sq_pack_w3.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.sq_rotate_quantize_variant.restype = C.c_int
        lib.sq_rotate_quantize_variant.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.sq_prepare_weights_variant.restype = C.c_int
        lib.sq_prepare_weights_variant.argtypes = [
            C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.sq_decode_layer_status.restype = C.c_int
        lib.sq_decode_layer_status.argtypes = [C.c_void_p, C.c_void_p]
        lib.sq_w4a4_gemm.restype = C.c_int
        lib.sq_w4a4_gemm.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.sq_prepare_weights.restype = C.c_int
        lib.sq_prepare_weights.argtypes = [
            C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.sq_debug_rotq_plan.restype = C.c_int32
        lib.sq_debug_rotq_plan.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 8
        lib.sq_debug_set_option.restype = C.c_int
        lib.sq_debug_set_option.argtypes = [C.c_int, C.c_int32]
        lib.sq_kron_factor.restype = C.c_int
        lib.sq_kron_factor.argtypes = [C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        lib.sq_build_rotation.restype = C.c_int
        lib.sq_build_rotation.argtypes = [
            C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.sq_build_rotation_workspace_bytes.restype = C.c_int64
        lib.sq_build_rotation_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        lib.sq_status_string.restype = C.c_char_p
        lib.sq_status_string.argtypes = [C.c_int]
        _lib = lib
    return _lib


def sq_status_string(code: int) -> str:
    return _load().sq_status_string(int(code)).decode()


# sq_debug_option of singlequant.h
SQ_DEBUG_GEMM_LAUNCH_SHAPE = 0
SQ_DEBUG_ROTQ_RING = 1
SQ_DEBUG_ROTQ_R1_IN_REGISTERS = 2
SQ_DEBUG_ROTQ_PLAIN_KERNEL = 3
SQ_DEBUG_DECODE_SPIN_LIMIT = 4
SQ_DEBUG_W4A16_LAUNCH_SHAPE = 5


def sq_debug_set_option(option: int, value: int) -> None:
    """Force a launch variant (test and tuning aid; 0 = the library decides)."""
    _check(_load().sq_debug_set_option(int(option), int(value)))


def _check(code: int) -> None:
    if code != SQ_OK:
        raise SQError(code, sq_status_string(code))


def _dev_ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _host(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def sq_rotate_quantize(X, giv_i, giv_j, giv_theta, R1, R2, Q, scales, xrot_dbg=None, stream=None) -> None:
    """X fp16 [T, K] (row stride = X.stride(0)); giv_* host sequences of equal length P;
    R1 fp16 [n1, n1]; R2 fp16 [n2, n2]; outputs Q uint8 [T, K/2], scales fp32 [T],
    optional xrot_dbg fp32 [T, K].  All tensors are device tensors owned by the caller."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    T, K = int(X.shape[0]), int(X.shape[1])
    ldx = int(X.stride(0)) if T > 1 else K
    code = _load().sq_rotate_quantize(
        _dev_ptr(X), T, K, ldx,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(R1), int(R1.shape[0]), _dev_ptr(R2), int(R2.shape[0]),
        _dev_ptr(Q), _dev_ptr(scales), _dev_ptr(xrot_dbg), _stream_handle(stream))
    _check(code)


def sq_rotate_quantize_variant(X, giv_i, giv_j, giv_theta, R1, R2, bits, clip_ratio, Q, scales, xrot_dbg=None,
                               stream=None) -> None:
    """sq_rotate_quantize with the quantizer at ``bits`` bits (2..4) and a clipping ratio in (0, 1]."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    T, K = int(X.shape[0]), int(X.shape[1])
    ldx = int(X.stride(0)) if T > 1 else K
    code = _load().sq_rotate_quantize_variant(
        _dev_ptr(X), T, K, ldx,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(R1), int(R1.shape[0]), _dev_ptr(R2), int(R2.shape[0]), int(bits), float(clip_ratio),
        _dev_ptr(Q), _dev_ptr(scales), _dev_ptr(xrot_dbg), _stream_handle(stream))
    _check(code)


def sq_prepared_rotation_bytes(n1: int, n2: int) -> int:
    return int(_load().sq_prepared_rotation_bytes(int(n1), int(n2)))


def sq_prepare_rotation(R1, R2, prepared, stream=None) -> None:
    """R1 fp16 [n1, n1], R2 fp16 [n2, n2]; prepared: any device tensor of at least
    sq_prepared_rotation_bytes(n1, n2) bytes, written here and passed to
    sq_rotate_quantize_prepared together with n1 and n2."""
    n1, n2 = int(R1.shape[0]), int(R2.shape[0])
    need = sq_prepared_rotation_bytes(n1, n2)
    if prepared is not None and need > 0 and prepared.numel() * prepared.element_size() < need:
        raise ValueError("prepared is smaller than sq_prepared_rotation_bytes")
    _check(_load().sq_prepare_rotation(_dev_ptr(R1), n1, _dev_ptr(R2), n2, _dev_ptr(prepared),
                                       _stream_handle(stream)))


def sq_rotate_quantize_prepared(X, giv_i, giv_j, giv_theta, prepared, n1, n2, Q, scales, xrot_dbg=None,
                                stream=None) -> None:
    """As sq_rotate_quantize, with the output of sq_prepare_rotation in place of R1 and R2."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    T, K = int(X.shape[0]), int(X.shape[1])
    ldx = int(X.stride(0)) if T > 1 else K
    need = sq_prepared_rotation_bytes(n1, n2)
    if prepared is not None and need > 0 and prepared.numel() * prepared.element_size() < need:
        raise ValueError("prepared is smaller than sq_prepared_rotation_bytes")
    code = _load().sq_rotate_quantize_prepared(
        _dev_ptr(X), T, K, ldx,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(prepared), int(n1), int(n2),
        _dev_ptr(Q), _dev_ptr(scales), _dev_ptr(xrot_dbg), _stream_handle(stream))
    _check(code)


def sq_w4a4_gemm(Qx, sx, Qw, sw, Y, acc_dbg=None, stream=None) -> None:
    """Qx uint8 [T, K/2], sx fp32 [T], Qw uint8 [N, K/2], sw fp32 [N]; output Y fp16 [T, N]
    (row stride = Y.stride(0)); optional acc_dbg int32 [T, N]."""
    T, Kh = int(Qx.shape[0]), int(Qx.shape[1])
    N = int(Qw.shape[0])
    ldy = int(Y.stride(0)) if T > 1 else max(N, 1)
    code = _load().sq_w4a4_gemm(
        _dev_ptr(Qx), _dev_ptr(sx), T, 2 * Kh, _dev_ptr(Qw), _dev_ptr(sw), N,
        _dev_ptr(Y), ldy, _dev_ptr(acc_dbg), _stream_handle(stream))
    _check(code)


def sq_decode_weights_bytes(K: int, N: int) -> int:
    return int(_load().sq_decode_weights_bytes(int(K), int(N)))


def sq_tile_weights_decode(Qw, Qw_tiled, stream=None) -> None:
    """Weight codes Qw uint8 [N, K/2] -> the decode layout in Qw_tiled (any uint8 device tensor of
    at least sq_decode_weights_bytes(K, N) bytes)."""
    N, K = int(Qw.shape[0]), 2 * int(Qw.shape[1])
    need = sq_decode_weights_bytes(K, N)
    if Qw_tiled is not None and Qw_tiled.numel() * Qw_tiled.element_size() < need:
        raise ValueError("Qw_tiled is smaller than sq_decode_weights_bytes")
    _check(_load().sq_tile_weights_decode(_dev_ptr(Qw), K, N, _dev_ptr(Qw_tiled), _stream_handle(stream)))


def sq_w4a4_gemm_decode(Qx, sx, Qw_tiled, sw, Y, acc_dbg=None, stream=None) -> None:
    """sq_w4a4_gemm for at most 32 tokens on weights in the decode layout; N = len(sw)."""
    T, Kh = int(Qx.shape[0]), int(Qx.shape[1])
    N = int(sw.shape[0])
    need = sq_decode_weights_bytes(2 * Kh, N)
    if Qw_tiled is not None and Qw_tiled.numel() * Qw_tiled.element_size() < need:
        raise ValueError("Qw_tiled is smaller than sq_decode_weights_bytes")
    ldy = int(Y.stride(0)) if T > 1 else max(N, 1)
    code = _load().sq_w4a4_gemm_decode(
        _dev_ptr(Qx), _dev_ptr(sx), T, 2 * Kh, _dev_ptr(Qw_tiled), _dev_ptr(sw), N,
        _dev_ptr(Y), ldy, _dev_ptr(acc_dbg), _stream_handle(stream))
    _check(code)


def sq_rotate_fp16(X, giv_i, giv_j, giv_theta, R1, R2, Xrot, stream=None) -> None:
    """Weight-only setting: the rotated rows as fp16, no quantizer.  X fp16 [T, K]; Xrot fp16
    [T, K] (row stride = Xrot.stride(0)); the rest as sq_rotate_quantize."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    T, K = int(X.shape[0]), int(X.shape[1])
    ldx = int(X.stride(0)) if T > 1 else K
    ldo = int(Xrot.stride(0)) if T > 1 else K
    code = _load().sq_rotate_fp16(
        _dev_ptr(X), T, K, ldx,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(R1), int(R1.shape[0]), _dev_ptr(R2), int(R2.shape[0]), _dev_ptr(Xrot), ldo, _stream_handle(stream))
    _check(code)


def sq_w4a16_gemm(X, Qw, sw, Y, stream=None) -> None:
    """Weight-only setting: X fp16 [T, K] times weight codes Qw uint8 [N, K/2] with steps sw
    fp32 [N] -> Y fp16 [T, N]."""
    T, K = int(X.shape[0]), int(X.shape[1])
    N = int(Qw.shape[0])
    ldx = int(X.stride(0)) if T > 1 else K
    ldy = int(Y.stride(0)) if T > 1 else max(N, 1)
    _check(_load().sq_w4a16_gemm(_dev_ptr(X), T, K, ldx, _dev_ptr(Qw), _dev_ptr(sw), N, _dev_ptr(Y), ldy,
                                 _stream_handle(stream)))


def sq_pack_w3(Qw, Qw3, stream=None) -> None:
    """Nibble codes Qw uint8 [N, K/2] (all in [-4, 3]) -> 3-bit storage Qw3 uint8 [N, 3K/8]."""
    N, K = int(Qw.shape[0]), 2 * int(Qw.shape[1])
    if Qw3 is not None and tuple(Qw3.shape) != (N, 3 * K // 8):
        raise ValueError("Qw3 must be [N, 3K/8]")
    _check(_load().sq_pack_w3(_dev_ptr(Qw), K, N, _dev_ptr(Qw3), _stream_handle(stream)))


def sq_w3a16_gemm(X, Qw3, sw, Y, stream=None) -> None:
    """sq_w4a16_gemm on weight codes in the 3-bit storage: Qw3 uint8 [N, 3K/8]."""
    T, K = int(X.shape[0]), int(X.shape[1])
    N = int(Qw3.shape[0])
    if int(Qw3.shape[1]) * 8 != 3 * K:
        raise ValueError("Qw3 must be [N, 3K/8]")
    ldx = int(X.stride(0)) if T > 1 else K
    ldy = int(Y.stride(0)) if T > 1 else max(N, 1)
    _check(_load().sq_w3a16_gemm(_dev_ptr(X), T, K, ldx, _dev_ptr(Qw3), _dev_ptr(sw), N, _dev_ptr(Y), ldy,
                                 _stream_handle(stream)))


def sq_decode_layer_workspace_bytes(T: int, K: int) -> int:
    return int(_load().sq_decode_layer_workspace_bytes(int(T), int(K)))


def sq_decode_layer(X, giv_i, giv_j, giv_theta, prepared, n1, n2, Qw, sw, Y, workspace, stream=None) -> None:
    """sq_rotate_quantize_prepared followed by sq_w4a4_gemm in one launch, for at most 32 tokens.
    workspace: device tensor of at least sq_decode_layer_workspace_bytes(T, K) bytes whose first
    16 bytes were zero before the first call (every call leaves them zero again)."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    T, K = int(X.shape[0]), int(X.shape[1])
    N = int(Qw.shape[0])
    ldx = int(X.stride(0)) if T > 1 else K
    ldy = int(Y.stride(0)) if T > 1 else max(N, 1)
    need = sq_decode_layer_workspace_bytes(T, K)
    if workspace is not None and need > 0 and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace is smaller than sq_decode_layer_workspace_bytes")
    need_p = sq_prepared_rotation_bytes(n1, n2)
    if prepared is not None and need_p > 0 and prepared.numel() * prepared.element_size() < need_p:
        raise ValueError("prepared is smaller than sq_prepared_rotation_bytes")
    code = _load().sq_decode_layer(
        _dev_ptr(X), T, K, ldx,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(prepared), int(n1), int(n2),
        _dev_ptr(Qw), _dev_ptr(sw), N, _dev_ptr(Y), ldy, _dev_ptr(workspace), _stream_handle(stream))
    _check(code)


def sq_decode_layer_status(workspace=None, stream=None) -> None:
    """Waits for the stream, then raises SQError (status 6) if a workgroup of any sq_decode_layer
    call on this workspace (None: the array inside the library) gave up its wait; clears the word."""
    _check(_load().sq_decode_layer_status(_dev_ptr(workspace), _stream_handle(stream)))


def sq_decode_layer_static(X, giv_i, giv_j, giv_theta, prepared, n1, n2, Qw, sw, Y, stream=None) -> None:
    """sq_decode_layer with the workspace inside the library (no device allocation anywhere on
    the way: the binding passes pointers of existing tensors only)."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    T, K = int(X.shape[0]), int(X.shape[1])
    N = int(Qw.shape[0])
    ldx = int(X.stride(0)) if T > 1 else K
    ldy = int(Y.stride(0)) if T > 1 else max(N, 1)
    need_p = sq_prepared_rotation_bytes(n1, n2)
    if prepared is not None and need_p > 0 and prepared.numel() * prepared.element_size() < need_p:
        raise ValueError("prepared is smaller than sq_prepared_rotation_bytes")
    code = _load().sq_decode_layer_static(
        _dev_ptr(X), T, K, ldx,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(prepared), int(n1), int(n2),
        _dev_ptr(Qw), _dev_ptr(sw), N, _dev_ptr(Y), ldy, _stream_handle(stream))
    _check(code)


def sq_prepare_weights(W, giv_i, giv_j, giv_theta, R1, R2, workspace, Qw, sw, stream=None) -> None:
    """W fp16 [K, N] (row stride = W.stride(0)); workspace fp16 with at least N*K elements;
    outputs Qw uint8 [N, K/2], sw fp32 [N].  Givens list and R1, R2 as in sq_rotate_quantize."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    K, N = int(W.shape[0]), int(W.shape[1])
    ldw = int(W.stride(0)) if K > 1 else max(N, 1)
    if workspace is not None and workspace.numel() < N * K:
        raise ValueError("workspace holds fewer than N*K elements")
    code = _load().sq_prepare_weights(
        _dev_ptr(W), K, N, ldw,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(R1), int(R1.shape[0]), _dev_ptr(R2), int(R2.shape[0]),
        _dev_ptr(workspace), _dev_ptr(Qw), _dev_ptr(sw), _stream_handle(stream))
    _check(code)


def sq_prepare_weights_variant(W, giv_i, giv_j, giv_theta, R1, R2, bits, clip_ratio, workspace, Qw, sw,
                               stream=None) -> None:
    """sq_prepare_weights with the quantizer at ``bits`` bits (2..4) and a clipping ratio in (0, 1]."""
    gi, gj, gt = _host(giv_i, np.int32), _host(giv_j, np.int32), _host(giv_theta, np.float32)
    P = 0 if gi is None else int(gi.size)
    K, N = int(W.shape[0]), int(W.shape[1])
    ldw = int(W.stride(0)) if K > 1 else max(N, 1)
    if workspace is not None and workspace.numel() < N * K:
        raise ValueError("workspace holds fewer than N*K elements")
    code = _load().sq_prepare_weights_variant(
        _dev_ptr(W), K, N, ldw,
        None if gi is None else gi.ctypes.data, None if gj is None else gj.ctypes.data,
        None if gt is None else gt.ctypes.data, P,
        _dev_ptr(R1), int(R1.shape[0]), _dev_ptr(R2), int(R2.shape[0]), int(bits), float(clip_ratio),
        _dev_ptr(workspace), _dev_ptr(Qw), _dev_ptr(sw), _stream_handle(stream))
    _check(code)


def sq_kron_factor(n: int):
    """Alg. 1: (n1, n2) with n = n1 * n2 and n2 the power of two closest to sqrt(n).  Host only."""
    a, b = C.c_int32(0), C.c_int32(0)
    _check(_load().sq_kron_factor(int(n), C.byref(a), C.byref(b)))
    return a.value, b.value


def sq_build_rotation_workspace_bytes(T: int, n1: int, n2: int) -> int:
    return int(_load().sq_build_rotation_workspace_bytes(int(T), int(n1), int(n2)))


def sq_build_rotation(X, n1, n2, giv_i, giv_j, giv_theta, R1, R2, workspace, stream=None) -> None:
    """X fp16 [T, K] calibration activations; outputs (all device tensors): giv_i, giv_j int32 [P],
    giv_theta fp32 [P] (P = their length; None for P = 0), R1 fp16 [n1, n1], R2 fp16 [n2, n2];
    workspace: any device tensor of at least sq_build_rotation_workspace_bytes(T, n1, n2) bytes."""
    T, K = int(X.shape[0]), int(X.shape[1])
    ldx = int(X.stride(0)) if T > 1 else K
    P = 0 if giv_i is None else int(giv_i.numel())
    need = sq_build_rotation_workspace_bytes(T, n1, n2)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace is smaller than sq_build_rotation_workspace_bytes")
    code = _load().sq_build_rotation(
        _dev_ptr(X), T, K, ldx, int(n1), int(n2), P, _dev_ptr(giv_i), _dev_ptr(giv_j), _dev_ptr(giv_theta),
        _dev_ptr(R1), _dev_ptr(R2), _dev_ptr(workspace), _stream_handle(stream))
    _check(code)
