"""Host-side checks of the C-ABI library that need no GPU: it loads, it exports every symbol the
header declares, and argument validation returns the documented codes before anything is
enqueued (the device pointers below are never dereferenced)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2511_22316_amd as sq
from paper_2511_22316_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sq.library_path()):
        from paper_2511_22316_amd import build
        build.build()
    return binding._load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "singlequant.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sq_[a-z0-9_]+)\s*\(", header))
    assert {"sq_rotate_quantize", "sq_w4a4_gemm", "sq_prepare_weights", "sq_status_string"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in singlequant.h but not exported"
    # and the other way round: no C symbol of the library's own prefix without a declaration
    import subprocess
    table = subprocess.run(["nm", "-D", "--defined-only", sq.library_path()], capture_output=True, text=True,
                           check=True).stdout
    exported = {line.split()[-1] for line in table.splitlines() if line.split()[-1].startswith("sq_")}
    assert exported and exported <= declared, f"exported but not declared: {sorted(exported - declared)}"


def test_binding_declares_the_argument_types_of_every_entry_point(lib):
    """A function called through ctypes without declared argument types gets its pointers cut to
    32 bits.  Every function the header declares has them in the binding, with as many entries as
    the declaration has parameters."""
    header = open(os.path.join(ROOT, "include", "singlequant.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    found = re.findall(r"\b(sq_[a-z0-9_]+)\s*\(([^;{]*?)\)\s*;", header, flags=re.S)
    assert len(found) >= 25
    for name, params in found:
        fn = getattr(lib, name)
        n_params = 0 if params.strip() in ("", "void") else params.count(",") + 1
        assert fn.argtypes is not None, f"{name}: argument types not declared in binding.py"
        assert len(fn.argtypes) == n_params, f"{name}: {len(fn.argtypes)} argument types for {n_params} parameters"


def test_status_strings(lib):
    texts = {sq.sq_status_string(c) for c in range(6)}
    assert len(texts) == 6 and sq.sq_status_string(0) == "ok"
    assert sq.sq_status_string(99) == "unknown status"


FAKE = 0x1000          # 16-byte aligned, never dereferenced: validation fails first


def _rq(lib, T=4, K=64, ldx=64, gi=(1,), gj=(2,), gt=(0.1,), n1=8, n2=8, X=FAKE, R1=FAKE, R2=FAKE,
        Q=FAKE, s=FAKE):
    gi_a, gj_a = np.asarray(gi, np.int32), np.asarray(gj, np.int32)
    gt_a = np.asarray(gt, np.float32)
    return lib.sq_rotate_quantize(X, T, K, ldx, gi_a.ctypes.data, gj_a.ctypes.data, gt_a.ctypes.data,
                                  len(gi_a), R1, n1, R2, n2, Q, s, None, None)


def test_rotate_quantize_argument_errors(lib):
    assert _rq(lib, K=63) == 2                      # K != n1*n2
    assert _rq(lib, n1=4, n2=16, K=65) == 2
    assert _rq(lib, T=-1) == 2
    assert _rq(lib, ldx=32) == 2                    # leading dimension shorter than a row
    assert _rq(lib, K=36, n1=9, n2=4, ldx=40) == 2  # n2 not a multiple of 8
    assert _rq(lib, K=129 * 8, n1=129, n2=8, ldx=129 * 8) == 2
    assert _rq(lib, gi=(64,)) == 3                  # index out of range
    assert _rq(lib, gi=(-1,)) == 3
    assert _rq(lib, gi=(5,), gj=(5,)) == 3          # i == j
    assert _rq(lib, X=None) == 1
    assert _rq(lib, R1=None) == 1
    assert _rq(lib, Q=None) == 1
    assert _rq(lib, X=FAKE + 2) == 4
    assert _rq(lib, ldx=68) == 4                    # rows not 16-byte aligned
    assert _rq(lib, T=0) == 0                       # nothing to do, nothing enqueued
    many = tuple(range(65))
    assert _rq(lib, gi=many, gj=tuple(i + 1 for i in many), gt=(0.0,) * 65, K=128, n1=8, n2=16, ldx=128) == 2


def _rqp(lib, T=4, K=64, ldx=64, gi=(1,), gj=(2,), gt=(0.1,), n1=8, n2=8, X=FAKE, prepared=FAKE, Q=FAKE, s=FAKE):
    gi_a, gj_a = np.asarray(gi, np.int32), np.asarray(gj, np.int32)
    gt_a = np.asarray(gt, np.float32)
    return lib.sq_rotate_quantize_prepared(X, T, K, ldx, gi_a.ctypes.data, gj_a.ctypes.data, gt_a.ctypes.data,
                                           len(gi_a), prepared, n1, n2, Q, s, None, None)


def test_prepared_rotation_argument_errors_and_sizes(lib):
    """The prepared variant validates like the plain one; nothing is dereferenced or enqueued."""
    assert _rqp(lib, K=63) == 2
    assert _rqp(lib, T=-1) == 2
    assert _rqp(lib, ldx=32) == 2
    assert _rqp(lib, K=36, n1=9, n2=4, ldx=40) == 2
    assert _rqp(lib, gi=(64,)) == 3
    assert _rqp(lib, gi=(5,), gj=(5,)) == 3
    assert _rqp(lib, prepared=None) == 1
    assert _rqp(lib, X=None) == 1
    assert _rqp(lib, prepared=FAKE + 8) == 4
    assert _rqp(lib, X=FAKE + 2) == 4
    assert _rqp(lib, T=0) == 0
    prep = lambda **kw: lib.sq_prepare_rotation(kw.get("R1", FAKE), kw.get("n1", 8), kw.get("R2", FAKE),
                                                kw.get("n2", 8), kw.get("out", FAKE), None)
    assert prep(n2=4) == 2 and prep(n1=129) == 2 and prep(n1=0) == 2
    assert prep(n1=128, n2=256) == 2                # K beyond the limit
    assert prep(R1=None) == 1 and prep(out=None) == 1
    assert prep(R2=FAKE + 4) == 4 and prep(out=FAKE + 2) == 4
    size = lib.sq_prepared_rotation_bytes
    # copies of R1 and R2 padded to 256 bytes, plus 1 KB per 32-column block and 16-row step of
    # each factor where the matrix-core kernel covers the shape
    assert size(8, 8) == 256 + 256
    assert size(64, 64) == 8192 + 8192 + (2 * 4 + 2 * 4) * 1024
    assert size(86, 128) == 14848 + 32768 + (3 * 6 + 4 * 8) * 1024
    assert size(128, 128) == 2 * 32768 + 2 * 4 * 8 * 1024
    assert size(9, 4) == 0 and size(0, 8) == 0 and size(128, 256) == 0


def _dl(lib, T=4, K=512, ldx=512, gi=(1,), gj=(2,), gt=(0.1,), n1=16, n2=32, X=FAKE, prepared=FAKE, Qw=FAKE, sw=FAKE,
        N=64, Y=FAKE, ldy=64, ws=FAKE - 0x1000 + 0x2000):
    gi_a, gj_a = np.asarray(gi, np.int32), np.asarray(gj, np.int32)
    gt_a = np.asarray(gt, np.float32)
    return lib.sq_decode_layer(X, T, K, ldx, gi_a.ctypes.data, gj_a.ctypes.data, gt_a.ctypes.data, len(gi_a),
                               prepared, n1, n2, Qw, sw, N, Y, ldy, ws, None)


def test_decode_layer_argument_errors_and_workspace_size(lib):
    assert _dl(lib, T=33) == 2                      # more tokens than the single launch takes
    assert _dl(lib, T=-1) == 2
    assert _dl(lib, K=500) == 2                     # K != n1*n2
    assert _dl(lib, K=64, n1=8, n2=8, ldx=64) == 2  # a shape only the two calls take
    assert _dl(lib, K=11008, n1=86, n2=128, ldx=11008) == 2
    assert _dl(lib, ldx=256) == 2
    assert _dl(lib, ldy=32) == 2
    assert _dl(lib, gi=(512,)) == 3
    assert _dl(lib, gi=(7,), gj=(7,)) == 3
    assert _dl(lib, prepared=None) == 1
    assert _dl(lib, X=None) == 1 and _dl(lib, Qw=None) == 1 and _dl(lib, Y=None) == 1 and _dl(lib, ws=None) == 1
    assert _dl(lib, X=FAKE + 2) == 4
    assert _dl(lib, ws=FAKE + 16) == 4              # workspace must be 256-byte aligned
    assert _dl(lib, Y=FAKE + 1) == 4
    assert _dl(lib, T=0) == 0 and _dl(lib, N=0) == 0
    size = lib.sq_decode_layer_workspace_bytes
    assert size(8, 8192) == 512 + 8 * 4096
    assert size(32, 512) == 512 + 32 * 256
    assert size(33, 512) == 0 and size(4, 0) == 0 and size(-1, 512) == 0


def test_decode_layer_static_argument_errors(lib):
    """The entry point with the workspace inside the library: the same checks in the same order
    (every case here returns before anything touches a device)."""
    def call(T=8, K=512, ldx=512, gi=(1,), gj=(2,), gt=(0.1,), prepared=FAKE, n1=16, n2=32, X=FAKE, Qw=FAKE, sw=FAKE,
             N=64, Y=FAKE, ldy=64):
        gi_a, gj_a, gt_a = np.asarray(gi, np.int32), np.asarray(gj, np.int32), np.asarray(gt, np.float32)
        return lib.sq_decode_layer_static(X, T, K, ldx, gi_a.ctypes.data, gj_a.ctypes.data, gt_a.ctypes.data,
                                          len(gi_a), prepared, n1, n2, Qw, sw, N, Y, ldy, None)
    assert call(T=33) == 2 and call(T=-1) == 2      # beyond what the array inside the library holds
    assert call(K=32768, n1=128, n2=256, ldx=32768) == 2
    assert call(K=500) == 2 and call(ldx=256) == 2 and call(ldy=32) == 2
    assert call(K=64, n1=8, n2=8, ldx=64) == 2
    assert call(gi=(512,)) == 3
    assert call(prepared=None) == 1 and call(X=None) == 1 and call(Qw=None) == 1 and call(Y=None) == 1
    assert call(X=FAKE + 2) == 4 and call(Y=FAKE + 1) == 4
    assert call(T=0) == 0 and call(N=0) == 0


def test_weight_only_argument_errors(lib):
    def rot(T=4, K=64, ldx=64, gi=(1,), gj=(2,), gt=(0.1,), n1=8, n2=8, X=FAKE, R1=FAKE, R2=FAKE, out=FAKE, ldo=64):
        gi_a, gj_a, gt_a = np.asarray(gi, np.int32), np.asarray(gj, np.int32), np.asarray(gt, np.float32)
        return lib.sq_rotate_fp16(X, T, K, ldx, gi_a.ctypes.data, gj_a.ctypes.data, gt_a.ctypes.data, len(gi_a),
                                  R1, n1, R2, n2, out, ldo, None)
    lib.sq_rotate_fp16.restype = C.c_int
    lib.sq_rotate_fp16.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64,
                                   C.c_void_p]
    assert rot(K=63) == 2 and rot(ldo=32) == 2 and rot(ldo=0) == 2 and rot(T=-1) == 2 and rot(ldx=8) == 2
    assert rot(gi=(64,)) == 3 and rot(gi=(2,)) == 3
    assert rot(out=None) == 1 and rot(X=None) == 1 and rot(R1=None) == 1
    assert rot(out=FAKE + 2) == 4 and rot(ldo=68) == 4 and rot(X=FAKE + 8) == 4
    assert rot(T=0) == 0

    def mm(T=4, K=64, ldx=64, N=8, ldy=8, X=FAKE, Qw=FAKE, sw=FAKE, Y=FAKE):
        return lib.sq_w4a16_gemm(X, T, K, ldx, Qw, sw, N, Y, ldy, None)
    lib.sq_w4a16_gemm.restype = C.c_int
    lib.sq_w4a16_gemm.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_void_p, C.c_int64, C.c_void_p]
    assert mm(K=96) == 2 and mm(K=0) == 2 and mm(T=-1) == 2 and mm(ldy=6) == 2 and mm(ldx=32) == 2 and mm(K=262144, ldx=262144) == 2
    assert mm(X=None) == 1 and mm(Qw=None) == 1 and mm(Y=None) == 1 and mm(sw=None) == 1
    assert mm(X=FAKE + 4) == 4 and mm(ldx=68) == 4 and mm(Qw=FAKE + 8) == 4 and mm(Y=FAKE + 1) == 4
    assert mm(T=0) == 0 and mm(N=0, ldy=0) == 0


def _gemm(lib, T=4, K=64, N=8, ldy=8, Qx=FAKE, sx=FAKE, Qw=FAKE, sw=FAKE, Y=FAKE):
    return lib.sq_w4a4_gemm(Qx, sx, T, K, Qw, sw, N, Y, ldy, None, None)


def test_gemm_argument_errors(lib):
    assert _gemm(lib, K=48) == 2                    # K not a multiple of 32
    assert _gemm(lib, K=0) == 2
    assert _gemm(lib, T=-1) == 2
    assert _gemm(lib, ldy=6) == 2
    assert _gemm(lib, K=262144) == 2
    assert _gemm(lib, K=131072) == 2                # 256 * 64 * K would be 2^31: one past the int32 accumulators
    assert _gemm(lib, K=131040, T=0) == 0           # the largest K the entry point takes
    assert _gemm(lib, Qx=None) == 1
    assert _gemm(lib, Y=None) == 1
    assert _gemm(lib, Qw=FAKE + 8) == 4
    assert _gemm(lib, T=0) == 0
    assert _gemm(lib, N=0, ldy=0) == 0


def test_decode_layout_argument_errors_and_sizes(lib):
    assert lib.sq_decode_weights_bytes(256, 33) == 64 * 128
    assert lib.sq_decode_weights_bytes(8192, 28672) == 28672 * 4096
    assert lib.sq_decode_weights_bytes(320, 8) == 0 and lib.sq_decode_weights_bytes(256, -1) == 0
    assert lib.sq_decode_weights_bytes(131072, 8) == 0

    def tile(K=256, N=8, Qw=FAKE, Qt=FAKE):
        return lib.sq_tile_weights_decode(Qw, K, N, Qt, None)
    assert tile(K=128) == 2 and tile(K=0) == 2 and tile(N=-1) == 2
    assert tile(Qw=None) == 1 and tile(Qt=None) == 1
    assert tile(Qw=FAKE + 8) == 4 and tile(Qt=FAKE + 4) == 4
    assert tile(N=0) == 0

    def mm(T=4, K=256, N=8, ldy=8, Qx=FAKE, sx=FAKE, Qt=FAKE, sw=FAKE, Y=FAKE):
        return lib.sq_w4a4_gemm_decode(Qx, sx, T, K, Qt, sw, N, Y, ldy, None, None)
    assert mm(T=33) == 2 and mm(K=128) == 2 and mm(K=288) == 2 and mm(T=-1) == 2 and mm(ldy=6) == 2
    assert mm(Qx=None) == 1 and mm(Qt=None) == 1 and mm(Y=None) == 1 and mm(sw=None) == 1
    assert mm(Qt=FAKE + 8) == 4 and mm(Y=FAKE + 1) == 4 and mm(sx=FAKE + 2) == 4
    assert mm(T=0) == 0 and mm(N=0, ldy=0) == 0


def test_variant_and_three_bit_argument_errors(lib):
    def rq(bits=4, clip=1.0, T=0, K=64):
        gi, gj, gt = np.asarray([1], np.int32), np.asarray([2], np.int32), np.asarray([0.1], np.float32)
        return lib.sq_rotate_quantize_variant(FAKE, T, K, K, gi.ctypes.data, gj.ctypes.data, gt.ctypes.data, 1,
                                              FAKE, 8, FAKE, 8, bits, clip, FAKE, FAKE, None, None)
    assert rq() == 0 and rq(bits=3) == 0 and rq(bits=2, clip=0.5) == 0
    assert rq(bits=1) == 2 and rq(bits=5) == 2 and rq(clip=0.0) == 2 and rq(clip=1.5) == 2 and rq(clip=float("nan")) == 2
    assert rq(K=63) == 2

    def pw(bits=3, clip=1.0, N=0, ws=FAKE):
        gi, gj, gt = np.asarray([1], np.int32), np.asarray([2], np.int32), np.asarray([0.1], np.float32)
        return lib.sq_prepare_weights_variant(FAKE, 64, N, max(N, 1), gi.ctypes.data, gj.ctypes.data, gt.ctypes.data, 1,
                                              FAKE, 8, FAKE, 8, bits, clip, ws, FAKE, FAKE, None)
    assert pw() == 0 and pw(bits=7) == 2 and pw(clip=-1.0) == 2

    def pack(K=64, N=8, Q=FAKE, Q3=FAKE):
        return lib.sq_pack_w3(Q, K, N, Q3, None)
    assert pack(K=32) == 2 and pack(K=0) == 2 and pack(N=-1) == 2 and pack(K=262144) == 2
    assert pack(Q=None) == 1 and pack(Q3=None) == 1 and pack(Q=FAKE + 8) == 4 and pack(Q3=FAKE + 4) == 4
    assert pack(N=0) == 0

    def mm(T=4, K=256, ldx=256, N=8, ldy=8, X=FAKE, Q3=FAKE, sw=FAKE, Y=FAKE):
        return lib.sq_w3a16_gemm(X, T, K, ldx, Q3, sw, N, Y, ldy, None)
    assert mm(K=320, ldx=320) == 2 and mm(K=0) == 2 and mm(T=-1) == 2 and mm(ldy=6) == 2 and mm(ldx=128) == 2
    assert mm(T=16 * 65535 + 1) == 2
    assert mm(X=None) == 1 and mm(Q3=None) == 1 and mm(Y=None) == 1 and mm(sw=None) == 1
    assert mm(X=FAKE + 4) == 4 and mm(ldx=260) == 4 and mm(Q3=FAKE + 4) == 4 and mm(Y=FAKE + 1) == 4
    assert mm(T=0) == 0 and mm(N=0, ldy=0) == 0


def test_binding_raises_on_error(lib):
    with pytest.raises(sq.SQError) as e:
        binding._check(lib.sq_w4a4_gemm(FAKE, FAKE, 4, 48, FAKE, FAKE, 8, FAKE, 8, None, None))
    assert e.value.code == 2


def _pw(lib, K=64, N=8, ldw=8, gi=(1,), gj=(2,), gt=(0.1,), n1=8, n2=8, W=FAKE, ws=FAKE, R1=FAKE, R2=FAKE,
        Qw=FAKE, sw=FAKE):
    gi_a, gj_a = np.asarray(gi, np.int32), np.asarray(gj, np.int32)
    gt_a = np.asarray(gt, np.float32)
    return lib.sq_prepare_weights(W, K, N, ldw, gi_a.ctypes.data, gj_a.ctypes.data, gt_a.ctypes.data,
                                  len(gi_a), R1, n1, R2, n2, ws, Qw, sw, None)


def test_prepare_weights_argument_errors(lib):
    assert _pw(lib, N=-1) == 2
    assert _pw(lib, ldw=4) == 2                     # leading dimension shorter than a row
    assert _pw(lib, K=63) == 2                      # K != n1*n2 (the row kernel's check)
    assert _pw(lib, gi=(64,)) == 3
    assert _pw(lib, W=None) == 1
    assert _pw(lib, ws=None) == 1
    assert _pw(lib, R2=None) == 1
    assert _pw(lib, Qw=None) == 1
    assert _pw(lib, ws=FAKE + 8) == 4
    assert _pw(lib, W=FAKE + 1) == 4
    assert _pw(lib, Qw=FAKE + 4) == 4
    assert _pw(lib, N=0) == 0                       # nothing to do, nothing enqueued


def test_debug_options(lib):
    lib.sq_debug_set_option.restype = C.c_int
    lib.sq_debug_set_option.argtypes = [C.c_int, C.c_int32]
    assert lib.sq_debug_set_option(6, 1) == 2 and lib.sq_debug_set_option(-1, 1) == 2     # unknown options
    for option in range(6):
        assert lib.sq_debug_set_option(option, 0) == 0
    # a forced shape never changes what is checked before the launch
    assert lib.sq_debug_set_option(0, 5) == 0 and _gemm(lib, K=48) == 2 and _gemm(lib, T=0) == 0
    assert lib.sq_debug_set_option(0, 0) == 0


# ------------------------------------------------------------------ launch plan of the Givens list -----

def _plan(lib, gi, gj, n2):
    gi, gj = np.asarray(gi, np.int32), np.asarray(gj, np.int32)
    P = len(gi)
    ns, nq = C.c_int32(), C.c_int32()
    arr = lambda: np.full(128, -1, np.int32)
    chan, qslot, qq, si, sj, lv = arr(), arr(), arr(), arr(), arr(), arr()
    fn = lib.sq_debug_rotq_plan
    fn.restype = C.c_int32
    fn.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p] + [C.c_void_p] * 6
    levels = fn(gi.ctypes.data, gj.ctypes.data, P, n2, C.addressof(ns), C.addressof(nq), chan.ctypes.data,
                qslot.ctypes.data, qq.ctypes.data, si.ctypes.data, sj.ctypes.data, lv.ctypes.data)
    return levels, ns.value, nq.value, chan, qslot, qq, si[:P], sj[:P], lv[:P]


@pytest.mark.parametrize("seed", range(12))
def test_givens_plan_keeps_list_order(lib, seed):
    """The regrouping into levels must be equivalent to the list: slots name the touched channels
    one to one, pairs of one level share no channel, and a pair sits in a later level than every
    earlier pair it shares a channel with."""
    g = np.random.default_rng(seed)
    n2 = int(g.choice([32, 64, 128]))
    K = n2 * int(g.choice([16, 64, 86]))
    P = int(g.integers(1, 65))
    pool = g.choice(K, size=int(g.integers(2, 2 * P + 1)), replace=False)     # small pools force reuse
    gi = g.choice(pool, size=P)
    gj = np.array([g.choice(pool[pool != a]) for a in gi])
    levels, n_slots, n_qslots, chan, qslot, qq, si, sj, lv = _plan(lib, gi, gj, n2)
    touched = sorted(set(gi.tolist()) | set(gj.tolist()))
    assert levels >= 1 and n_slots == len(touched)
    assert sorted(chan[:n_slots].tolist()) == touched
    assert n_qslots == len({c % n2 for c in touched})
    assert all(qq[qslot[s]] == chan[s] % n2 for s in range(n_slots))
    assert all(chan[si[p]] == gi[p] and chan[sj[p]] == gj[p] for p in range(P))
    assert lv.min() == 0 and lv.max() == levels - 1
    for l in range(levels):
        used = [c for p in range(P) if lv[p] == l for c in (gi[p], gj[p])]
        assert len(used) == len(set(used)), "pairs of one level share a channel"
    last = {}
    for p in range(P):                                  # dependencies point to earlier levels
        for c in (gi[p], gj[p]):
            if c in last:
                assert lv[p] > last[c]
        last[gi[p]] = last[gj[p]] = lv[p]
    # and no pair is pushed later than its dependencies force it to be
    last = {}
    for p in range(P):
        need = 1 + max(last.get(gi[p], -1), last.get(gj[p], -1))
        assert lv[p] == need
        last[gi[p]] = last[gj[p]] = lv[p]


def test_givens_plan_limits(lib):
    levels, n_slots, n_qslots, *_ = _plan(lib, [], [], 64)
    assert (levels, n_slots, n_qslots) == (0, 0, 0)
    gi = np.arange(64) * 128                     # 128 channels in 128 different columns of an n2 = 128 view
    gj = np.arange(64) * 128 + 64 + np.arange(64)
    gi = gi + np.arange(64)
    levels, n_slots, n_qslots, *_ = _plan(lib, gi, gj, 128)
    assert levels == 1 and n_slots == 128 and n_qslots == 128


# ------------------------------------------------------------------ rotation constructor ---

def _br(lib, T=4, K=128, ldx=128, n1=8, n2=16, P=2, X=FAKE, gi=FAKE, gj=FAKE, gt=FAKE, R1=FAKE, R2=FAKE,
        ws=FAKE):
    return lib.sq_build_rotation(X, T, K, ldx, n1, n2, P, gi, gj, gt, R1, R2, ws, None)


def test_build_rotation_argument_errors(lib):
    assert _br(lib, X=None) == 1
    assert _br(lib, R2=None) == 1
    assert _br(lib, ws=None) == 1
    assert _br(lib, gi=None) == 1                   # P > 0 needs the three output lists
    assert _br(lib, T=0) == 2                       # a calibration batch cannot be empty
    assert _br(lib, K=120) == 2                     # K != n1*n2
    assert _br(lib, n1=16, n2=8, K=128, P=65) == 2
    assert _br(lib, n1=1, n2=128) == 2              # a URT needs at least two entries
    assert _br(lib, n1=4, n2=24, K=96, ldx=96) == 2  # n2 must be a power of two (Hadamard factor)
    assert _br(lib, n1=32, n2=4) == 2
    assert _br(lib, ldx=64) == 2
    assert _br(lib, n1=128, n2=256, K=32768, ldx=32768) == 2
    assert _br(lib, X=FAKE + 4) == 4
    assert _br(lib, ldx=132) == 4
    assert _br(lib, ws=FAKE + 8) == 4


def test_build_rotation_workspace_size(lib):
    f = sq.sq_build_rotation_workspace_bytes
    assert f(0, 8, 8) == 0 and f(4, 0, 8) == 0 and f(4, 129, 8) == 0 and f(4, 8, 257) == 0
    small, big = f(1, 64, 64), f(100000, 64, 64)
    assert small % 4 == 0 and small >= 4 * (1 + 2 * 64 * 64 + 3 * 64 * 64)
    assert big - small >= 4 * 99999 - 256           # one float per calibration row


def test_kron_factor_follows_alg1(lib, oracle):
    """Against the oracle's own routine and a brute force over every divisor that is a power of two."""
    for n in list(range(1, 300)) + [512, 4096, 5120, 8192, 11008, 13824, 14336, 16384, 28672, 2 ** 20 + 2 ** 10]:
        n1, n2 = sq.sq_kron_factor(n)
        assert n1 * n2 == n and (n2 & (n2 - 1)) == 0
        cands = [2 ** k for k in range(0, 31) if 2 ** k <= n and n % 2 ** k == 0]
        best = min(cands, key=lambda a: (abs(a - np.sqrt(n)), a))
        assert n2 == best
        assert (n1, n2) == tuple(oracle.kron_factor(n))
    assert sq.sq_kron_factor(4096) == (64, 64) and sq.sq_kron_factor(11008) == (86, 128)
    a = C.c_int32(0)
    assert lib.sq_kron_factor(0, C.byref(a), C.byref(a)) == 2
    assert lib.sq_kron_factor(8, None, C.byref(a)) == 1
