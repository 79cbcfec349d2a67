"""GPU parity of the quantizer variants (b bits, clipping ratio) and of the 3-bit weight storage
with its GEMM, through the C ABI against the CPU oracle.

Bars.  Steps and codes of the variant quantizer: those of the 4-bit path (steps within 1e-5
relative, every code within one level, at most 1e-4 of them different), plus: codes inside
[-2^(b-1), 2^(b-1) - 1]; where every quotient is exact in fp32 the codes EQUAL the oracle's.
3-bit storage: bit-exact.  W3A16 GEMM: the bound of the W4A16 GEMM (one fp16 spacing at the
oracle's value plus the fp32 summation slack), and -- the summation order being that of the
decode-shaped W4A16 kernel -- the same bits as sq_w4a16_gemm on the same codes kept as nibbles."""
import numpy as np
import pytest

from paper_2511_22316_amd import synth
from parity_util import CODE_FLIP_FRACTION, SCALE_TOL, codes_of, dev, host
from test_gpu_w4a16 import check_w4a16, run_w4a16

pytestmark = pytest.mark.gpu


def run_variant(L, bits, clip, X=None, want_xrot=False):
    import torch
    import paper_2511_22316_amd as sq
    X = L.X if X is None else X
    T, K = X.shape
    Q = torch.full((T, K // 2), 0x5A, dtype=torch.uint8, device="cuda")
    s = torch.full((T,), -1.0, dtype=torch.float32, device="cuda")
    xr = torch.empty((T, K), dtype=torch.float32, device="cuda") if want_xrot else None
    sq.sq_rotate_quantize_variant(dev(X), L.giv_i, L.giv_j, L.giv_theta, dev(L.R1), dev(L.R2), bits, clip, Q, s, xr)
    torch.cuda.synchronize()
    return host(Q), host(s), (host(xr) if want_xrot else None)


def check_variant_codes(Qg, sg, Qo, so, bits):
    rel = np.abs(sg.astype(np.float64) - so) / so
    assert rel.max() <= SCALE_TOL, f"steps: worst relative error {rel.max():.3e}"
    qg, qo = codes_of(Qg), codes_of(Qo)
    assert qg.min() >= -(2 ** (bits - 1)) and qg.max() <= 2 ** (bits - 1) - 1
    diff = np.abs(qg - qo)
    assert diff.max() <= 1, "a code differs by more than one level"
    frac = float(np.count_nonzero(diff)) / diff.size
    assert frac <= CODE_FLIP_FRACTION, f"{frac:.3e} of the codes differ"
    return frac


GENERIC = synth.LayerConfig("var_12x8", 9, 12, 8, 16, 3, "normal", 1, 50.0, 0.02, 20.0, 0.02, 78)
FOUR_BLOCKS = synth.LayerConfig("var_128x64", 19, 128, 64, 16, 12, "normal", 2, 80.0, 0.02, 20.0, 0.02, 79)


@pytest.mark.parametrize("bits,clip", [(3, 1.0), (4, 0.7), (3, 0.5), (2, 1.0), (4, 0.999)])
@pytest.mark.parametrize("name,T", [("tiny", 16), ("attn_proj", 70), ("mlp_down", 37), ("large_prefill", 33),
                                    ("generic", 9), ("four_blocks", 19)])
def test_variant_quantizer_matches_oracle(oracle, name, T, bits, clip):
    print(f"case variant quantizer {name} T={T} bits={bits} clip={clip}", flush=True)
    cfg = {"generic": GENERIC, "four_blocks": FOUR_BLOCKS}.get(name) or synth.CONFIGS[name]
    L = synth.layer(cfg, T)
    Qg, sg, xg = run_variant(L, bits, clip, want_xrot=True)
    xo = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Qo, so = oracle.quantize_rows_variant(xo, bits, clip)
    frac = check_variant_codes(Qg, sg, Qo, so, bits)
    qo = codes_of(Qo)
    clipped = float(np.mean((qo == 2 ** (bits - 1) - 1) | (qo == -(2 ** (bits - 1)))))
    print(f"  {frac:.2e} of the codes differ; {clipped:.3f} of them sit on an end level", flush=True)
    # the rotated rows do not depend on the quantizer: same bits as the plain call writes
    import torch
    import paper_2511_22316_amd as sq
    Q4 = torch.empty((T, cfg.K // 2), dtype=torch.uint8, device="cuda")
    s4 = torch.empty((T,), dtype=torch.float32, device="cuda")
    x4 = torch.empty((T, cfg.K), dtype=torch.float32, device="cuda")
    sq.sq_rotate_quantize(dev(L.X), L.giv_i, L.giv_j, L.giv_theta, dev(L.R1), dev(L.R2), Q4, s4, x4)
    torch.cuda.synchronize()
    assert np.array_equal(host(x4), xg)


@pytest.mark.parametrize("name,T", [("tiny", 16), ("attn_proj", 40), ("mlp_down", 20), ("generic", 9)])
def test_variant_with_four_bits_and_no_clipping_is_the_plain_call(oracle, name, T):
    print(f"case variant == plain {name}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = GENERIC if name == "generic" else synth.CONFIGS[name]
    L = synth.layer(cfg, T)
    Qv, sv, _ = run_variant(L, 4, 1.0)
    Q4 = torch.empty((T, cfg.K // 2), dtype=torch.uint8, device="cuda")
    s4 = torch.empty((T,), dtype=torch.float32, device="cuda")
    sq.sq_rotate_quantize(dev(L.X), L.giv_i, L.giv_j, L.giv_theta, dev(L.R1), dev(L.R2), Q4, s4)
    torch.cuda.synchronize()
    assert np.array_equal(host(Q4), Qv) and np.array_equal(host(s4), sv)


@pytest.mark.parametrize("n1,n2", [(16, 32), (64, 64), (64, 128), (86, 128), (128, 64), (12, 8)])
@pytest.mark.parametrize("bits,clip,top", [(4, 0.5, 14.0), (3, 0.75, 4.0), (3, 1.0, 3.0), (4, 0.25, 28.0), (2, 0.5, 2.0)])
def test_clipping_and_levels_on_exact_rows(oracle, n1, n2, bits, clip, top):
    """Identity rotation, no list, rows of multiples of 1/2 whose maximum is `top`: the step
    clip * top / (2^(b-1) - 1) is 1 exactly, every quotient is exact, and the codes must EQUAL the
    oracle's -- ties go up, what lies beyond the end levels is clamped to them."""
    print(f"case exact clipping {n1}x{n2} bits={bits} clip={clip}", flush=True)
    K = n1 * n2
    g = np.random.default_rng(n1 + n2 + bits)
    X = (g.integers(-int(2 * top), int(2 * top) + 1, size=(9, K)) / 2.0)
    X[:, 0] = [top, -top, top, -top, top, -top, top, -top, top]
    X[3, 1:] = np.clip(X[3, 1:], -1.0, 1.0)            # a row that only its maximum makes clip
    X = X.astype(np.float16)
    cfg = synth.LayerConfig(f"clip_{n1}x{n2}", 9, n1, n2, 8, 0, "normal", 0, 1.0, 0.0, 1.0, 0.02, 1)
    e = np.zeros(0, np.int32)
    Li = synth.Layer(cfg, X, e, e, np.zeros(0, np.float32), np.eye(n1, dtype=np.float16),
                     np.eye(n2, dtype=np.float16), None, None)
    Qg, sg, xg = run_variant(Li, bits, clip, want_xrot=True)
    assert np.array_equal(xg, X.astype(np.float32))
    Qo, so = oracle.quantize_rows_variant(X.astype(np.float64), bits, clip)
    assert np.all(so == 1.0) and np.array_equal(sg, so)
    assert np.array_equal(Qg, Qo)
    hi, lo = 2 ** (bits - 1) - 1, -(2 ** (bits - 1))
    want = np.clip(np.floor(X.astype(np.float64) + 0.5), lo, hi).astype(np.int16)
    assert np.array_equal(codes_of(Qg), want)
    if clip < 1.0:                      # the rows do reach beyond the end levels
        assert np.count_nonzero(X.astype(np.float64) >= hi + 0.5) > 9
        if top > 0.5 - lo:
            assert np.count_nonzero(X.astype(np.float64) < lo - 0.5) > 9


@pytest.mark.parametrize("name,N,bits,clip", [("tiny", 130, 3, 1.0), ("attn_proj", 200, 3, 0.8), ("tiny", 512, 4, 0.6)])
def test_prepare_weights_variant_matches_oracle(oracle, name, N, bits, clip):
    print(f"case prepare_weights_variant {name} N={N} bits={bits} clip={clip}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg, 16)
    Wt = synth.weights_t(cfg, N)
    W = torch.from_numpy(np.ascontiguousarray(Wt.T)).cuda()
    ws = torch.empty((N * cfg.K,), dtype=torch.float16, device="cuda")
    Qw = torch.empty((N, cfg.K // 2), dtype=torch.uint8, device="cuda")
    sw = torch.empty((N,), dtype=torch.float32, device="cuda")
    R1, R2 = dev(L.R1), dev(L.R2)
    sq.sq_prepare_weights_variant(W, L.giv_i, L.giv_j, L.giv_theta, R1, R2, bits, clip, ws, Qw, sw)
    torch.cuda.synchronize()
    Qo, so = oracle.prepare_weights_variant(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2, bits, clip)
    check_variant_codes(host(Qw), host(sw), Qo, so, bits)
    Lw = synth.Layer(cfg, Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2, None, None)
    Q2, s2, _ = run_variant(Lw, bits, clip)
    assert np.array_equal(Q2, host(Qw)) and np.array_equal(s2, host(sw))


def test_variant_arguments_are_checked():
    print("case variant argument checks", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    L = synth.layer(synth.CONFIGS["tiny"])
    T, K = L.X.shape
    Q = torch.empty((T, K // 2), dtype=torch.uint8, device="cuda")
    s = torch.empty((T,), dtype=torch.float32, device="cuda")
    for bits, clip in [(1, 1.0), (5, 1.0), (4, 0.0), (4, -0.5), (4, 1.0001), (3, float("nan"))]:
        with pytest.raises(sq.SQError) as e:
            sq.sq_rotate_quantize_variant(dev(L.X), L.giv_i, L.giv_j, L.giv_theta, dev(L.R1), dev(L.R2), bits, clip, Q, s)
        assert e.value.code == 2
    ws = torch.empty((K * 8,), dtype=torch.float16, device="cuda")
    with pytest.raises(sq.SQError) as e:
        sq.sq_prepare_weights_variant(torch.zeros((K, 8), dtype=torch.float16, device="cuda"), L.giv_i, L.giv_j,
                                      L.giv_theta, dev(L.R1), dev(L.R2), 7, 1.0, ws,
                                      torch.empty((8, K // 2), dtype=torch.uint8, device="cuda"),
                                      torch.empty((8,), dtype=torch.float32, device="cuda"))
    assert e.value.code == 2
    x = torch.zeros((4, 320), dtype=torch.float16, device="cuda")
    with pytest.raises(sq.SQError) as e:                 # K % 256 != 0
        sq.sq_w3a16_gemm(x, torch.zeros((8, 120), dtype=torch.uint8, device="cuda"),
                         torch.ones((8,), dtype=torch.float32, device="cuda"),
                         torch.empty((4, 8), dtype=torch.float16, device="cuda"))
    assert e.value.code == 2
    with pytest.raises(sq.SQError) as e:                 # K % 64 != 0
        sq.sq_pack_w3(torch.zeros((8, 48), dtype=torch.uint8, device="cuda"),
                      torch.zeros((8, 36), dtype=torch.uint8, device="cuda"))
    assert e.value.code == 2


# ------------------------------------------------------------------ 3-bit storage and GEMM --

def three_bit_codes(N, K, seed):
    c = np.random.default_rng(seed).integers(-4, 4, size=(N, K))
    nib = (c & 0xF).astype(np.uint8)
    return np.ascontiguousarray(nib[:, 0::2] | (nib[:, 1::2] << 4))


def run_pack_w3(Q):
    import torch
    import paper_2511_22316_amd as sq
    N, Kh = Q.shape
    out = torch.full((N, 3 * Kh // 4 + 8), 0xA5, dtype=torch.uint8, device="cuda")
    body = out.view(-1)[: N * (3 * Kh // 4)].view(N, 3 * Kh // 4)
    sq.sq_pack_w3(dev(Q), body)
    torch.cuda.synchronize()
    assert torch.all(out.view(-1)[N * (3 * Kh // 4):] == 0xA5), "sq_pack_w3 wrote past the end"
    return host(body)


@pytest.mark.parametrize("N,K", [(1, 64), (7, 192), (130, 512), (33, 8192), (1000, 1024)])
def test_pack_w3_bit_exact(oracle, N, K):
    print(f"case pack_w3 N={N} K={K}", flush=True)
    Q = three_bit_codes(N, K, N + K)
    got = run_pack_w3(Q)
    assert np.array_equal(got, oracle.pack_w3(Q))
    assert np.array_equal(oracle.unpack_w3(got), Q)


def run_w3a16(X, Q3, sw, ldy=None):
    import torch
    import paper_2511_22316_amd as sq
    T, N = X.shape[0], Q3.shape[0]
    Y = torch.full((T, ldy or N), -9.0, dtype=torch.float16, device="cuda")
    sq.sq_w3a16_gemm(dev(X), dev(Q3), dev(sw), Y[:, :N])
    torch.cuda.synchronize()
    return host(Y)


@pytest.mark.parametrize("T,K,N", [(1, 256, 1), (8, 1024, 24700), (32, 768, 10300), (20, 256, 50), (16, 8192, 300),
                                   (17, 2048, 33), (1, 4096, 4096), (40, 512, 100), (100, 256, 31), (8, 11008, 70)])
def test_w3a16_gemm_random_operands(oracle, T, K, N):
    print(f"case w3a16 gemm random T={T} K={K} N={N}", flush=True)
    g = np.random.default_rng(T + 3 * K + 5 * N)
    X = (g.standard_normal((T, K)) * g.choice([0.1, 1.0, 30.0], size=(T, 1))).astype(np.float16)
    Q = three_bit_codes(N, K, 500 + N)
    Q3 = run_pack_w3(Q)
    sw = g.uniform(1e-4, 5e-3, N).astype(np.float32)
    Yo, m = oracle.gemm_w3a16(X, Q3, sw, want_abs_sum=True)
    Yg = run_w3a16(X, Q3, sw, ldy=N + 3)
    check_w4a16(Yg[:, :N], Yo, m, K)
    assert np.all(Yg[:, N:] == -9.0)
    if T <= 32:
        # same kernel, same order of additions as the decode-shaped W4A16 kernel on the nibbles
        assert np.array_equal(Yg[:, :N], run_w4a16(X, Q, sw))
    # exactly representable case: equal bits
    Xi = g.integers(-3, 4, size=(T, K)).astype(np.float16)
    s4 = np.full(N, 0.25, np.float32)
    Yi = oracle.gemm_w3a16(Xi, Q3, s4)
    if np.max(np.abs(Yi.astype(np.float64))) < 2048:
        assert np.array_equal(run_w3a16(Xi, Q3, s4), Yi)


def test_w3a16_gemm_strided_input_and_empty(oracle):
    print("case w3a16 gemm strided input, empty", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    g = np.random.default_rng(41)
    T, K, N = 9, 512, 40
    X = g.standard_normal((T, K)).astype(np.float16)
    Q3 = oracle.pack_w3(three_bit_codes(N, K, 6))
    sw = np.full(N, 0.01, np.float32)
    Yo, m = oracle.gemm_w3a16(X, Q3, sw, want_abs_sum=True)
    wide = torch.full((T, K + 24), 1000.0, dtype=torch.float16, device="cuda")
    wide[:, :K] = dev(X)
    Y = torch.full((T, N + 5), -9.0, dtype=torch.float16, device="cuda")
    sq.sq_w3a16_gemm(wide[:, :K], dev(Q3), dev(sw), Y[:, :N])
    torch.cuda.synchronize()
    check_w4a16(host(Y)[:, :N], Yo, m, K)
    assert np.all(host(Y)[:, N:] == -9.0)
    sq.sq_w3a16_gemm(wide[:0, :K], dev(Q3), dev(sw), Y[:0, :N])
    sq.sq_pack_w3(torch.empty((0, K // 2), dtype=torch.uint8, device="cuda"),
                  torch.empty((0, 3 * K // 8), dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("name,T,N", [("tiny", 16, 512), ("attn_proj", 24, 300), ("decode", 8, 200)])
def test_w3a16_layer_end_to_end(oracle, name, T, N):
    """GPU pipeline (rotation to fp16, weight path at three bits, 3-bit storage, W3A16 GEMM) against
    the oracle pipeline; and three bits cost accuracy against four."""
    print(f"case W3A16 layer {name} T={T} N={N}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    from parity_util import Y_ROW_TOL
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg, T)
    Wt = synth.weights_t(cfg, N)
    xo = oracle.rotate_f16(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Qwo, swo = oracle.prepare_weights_variant(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2, 3, 1.0)
    Yo = oracle.gemm_w3a16(xo, oracle.pack_w3(Qwo), swo).astype(np.float64)
    dR1, dR2 = dev(L.R1), dev(L.R2)
    W = torch.from_numpy(np.ascontiguousarray(Wt.T)).cuda()
    ws = torch.empty((N * cfg.K,), dtype=torch.float16, device="cuda")
    Qw = torch.empty((N, cfg.K // 2), dtype=torch.uint8, device="cuda")
    sw = torch.empty((N,), dtype=torch.float32, device="cuda")
    sq.sq_prepare_weights_variant(W, L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, 3, 1.0, ws, Qw, sw)
    Qw3 = torch.empty((N, 3 * cfg.K // 8), dtype=torch.uint8, device="cuda")
    sq.sq_pack_w3(Qw, Qw3)
    Xr = torch.empty((T, cfg.K), dtype=torch.float16, device="cuda")
    sq.sq_rotate_fp16(dev(L.X), L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, Xr)
    Y = torch.empty((T, N), dtype=torch.float16, device="cuda")
    sq.sq_w3a16_gemm(Xr, Qw3, sw, Y)
    torch.cuda.synchronize()
    rel = np.linalg.norm(host(Y).astype(np.float64) - Yo, axis=1) / np.linalg.norm(Yo, axis=1)
    print(f"  worst row error {rel.max():.3e}", flush=True)
    assert rel.max() <= Y_ROW_TOL
    ref = L.X.astype(np.float64) @ Wt.astype(np.float64).T
    e3 = np.linalg.norm(host(Y).astype(np.float64) - ref) / np.linalg.norm(ref)
    Q4 = torch.empty_like(Qw)
    s4 = torch.empty_like(sw)
    sq.sq_prepare_weights(W, L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, ws, Q4, s4)
    Y4 = torch.empty_like(Y)
    sq.sq_w4a16_gemm(Xr, Q4, s4, Y4)
    torch.cuda.synchronize()
    e4 = np.linalg.norm(host(Y4).astype(np.float64) - ref) / np.linalg.norm(ref)
    print(f"  error against X W: W3A16 {e3:.3f}, W4A16 {e4:.3f}", flush=True)
    assert e4 < e3 < 0.5


# ------------------------------------------------------ decode layout of the W4A4 weights --

def run_tile_decode(Qw):
    import torch
    import paper_2511_22316_amd as sq
    N, Kh = Qw.shape
    need = sq.sq_decode_weights_bytes(2 * Kh, N)
    assert need == ((N + 31) // 32) * 32 * Kh
    out = torch.full((need + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    sq.sq_tile_weights_decode(dev(Qw), out[:need])
    torch.cuda.synchronize()
    assert torch.all(out[need:] == 0xA5), "sq_tile_weights_decode wrote past its stated size"
    return out[:need]


@pytest.mark.parametrize("N,K", [(1, 256), (33, 512), (100, 1024), (300, 8192), (4096, 768)])
def test_tile_weights_decode_bit_exact(oracle, N, K):
    print(f"case tile_weights_decode N={N} K={K}", flush=True)
    Qw = synth.random_codes(N, K, N + K)
    got = host(run_tile_decode(Qw))
    assert np.array_equal(got, oracle.tile_weights_decode(Qw))
    assert np.array_equal(oracle.untile_weights_decode(got, N, K), Qw)


@pytest.mark.parametrize("T,K,N", [(1, 256, 33), (8, 1024, 520), (32, 768, 8200), (16, 512, 10300), (31, 512, 24600),
                                   (8, 8192, 25000), (15, 8192, 700), (5, 2304, 12000), (16, 8192, 700),
                                   (32, 8192, 300), (20, 4096, 10300), (17, 4096, 24700), (3, 256, 31)])
def test_gemm_decode_layout_bit_exact(oracle, T, K, N):
    """sq_w4a4_gemm_decode on the tiled copy: accumulators equal to the oracle's, and accumulators
    and Y equal, bit for bit, to sq_w4a4_gemm on the canonical codes; every launch shape of the
    decode-shaped kernel, token rows in LDS and not, ragged channel tails (padded last block)."""
    print(f"case gemm decode layout T={T} K={K} N={N}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    Qx, Qw = synth.random_codes(T, K, 7 * T + K), synth.random_codes(N, K, 11 * N + K)
    g = np.random.default_rng(T + K + N)
    sx, sw = g.uniform(0.01, 2.0, T).astype(np.float32), g.uniform(1e-3, 1e-2, N).astype(np.float32)
    Qt = run_tile_decode(Qw)
    Y = torch.full((T, N + 3), -9.0, dtype=torch.float16, device="cuda")
    acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
    sq.sq_w4a4_gemm_decode(dev(Qx), dev(sx), Qt, dev(sw), Y[:, :N], acc)
    Y0 = torch.empty((T, N), dtype=torch.float16, device="cuda")
    acc0 = torch.empty((T, N), dtype=torch.int32, device="cuda")
    sq.sq_w4a4_gemm(dev(Qx), dev(sx), dev(Qw), dev(sw), Y0, acc0)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc0) and torch.equal(Y[:, :N], Y0)
    assert torch.all(Y[:, N:] == -9.0)
    _, acco = oracle.gemm(Qx, sx, Qw, sw)
    assert np.array_equal(host(acc), acco)


def test_gemm_decode_layout_full_size_decode_workload(oracle):
    """The decode workload at full size in the configuration the benchmark times (prepared rotation,
    then sq_w4a4_gemm_decode on the tiled weights): Y equal to sq_w4a4_gemm's, sampled accumulators
    computed one by one by the oracle."""
    print("case gemm decode layout, decode workload at full size", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS["decode"]
    L = synth.layer(cfg)
    T, K, N = cfg.T, cfg.K, cfg.N
    Qw = synth.random_codes(N, K, 4242)
    sw = np.random.default_rng(5).uniform(1e-3, 1e-2, N).astype(np.float32)
    dR1, dR2 = dev(L.R1), dev(L.R2)
    prepared = torch.empty((sq.sq_prepared_rotation_bytes(cfg.n1, cfg.n2),), dtype=torch.uint8, device="cuda")
    sq.sq_prepare_rotation(dR1, dR2, prepared)
    Qx = torch.empty((T, K // 2), dtype=torch.uint8, device="cuda")
    sx = torch.empty((T,), dtype=torch.float32, device="cuda")
    sq.sq_rotate_quantize_prepared(dev(L.X), L.giv_i, L.giv_j, L.giv_theta, prepared, cfg.n1, cfg.n2, Qx, sx)
    dQw, dsw = dev(Qw), dev(sw)
    Qt = run_tile_decode(Qw)
    Y = torch.empty((T, N), dtype=torch.float16, device="cuda")
    acc = torch.empty((T, N), dtype=torch.int32, device="cuda")
    sq.sq_w4a4_gemm_decode(Qx, sx, Qt, dsw, Y, acc)
    Y0 = torch.empty_like(Y)
    sq.sq_w4a4_gemm(Qx, sx, dQw, dsw, Y0)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y0)
    hQx, hacc = host(Qx), host(acc)
    g = np.random.default_rng(77)
    for t, n in zip(g.integers(0, T, 200), np.concatenate([[0, N - 1, 31, 32, N - 32], g.integers(0, N, 195)])):
        assert hacc[t, n] == oracle.gemm_acc_at(hQx, Qw, int(t), int(n))


def test_gemm_decode_layout_arguments_are_checked():
    print("case gemm decode layout argument checks", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    assert sq.sq_decode_weights_bytes(320, 8) == 0 and sq.sq_decode_weights_bytes(256, 33) == 64 * 128
    Qx = torch.zeros((33, 128), dtype=torch.uint8, device="cuda")
    sx = torch.ones((33,), dtype=torch.float32, device="cuda")
    Qt = torch.zeros((32 * 128,), dtype=torch.uint8, device="cuda")
    sw = torch.ones((8,), dtype=torch.float32, device="cuda")
    Y = torch.empty((33, 8), dtype=torch.float16, device="cuda")
    with pytest.raises(sq.SQError) as e:                    # 33 tokens
        sq.sq_w4a4_gemm_decode(Qx, sx, Qt, sw, Y)
    assert e.value.code == 2
    with pytest.raises(sq.SQError) as e:                    # K = 160
        sq.sq_w4a4_gemm_decode(Qx[:4, :80].contiguous(), sx[:4], Qt, sw, Y[:4])
    assert e.value.code == 2
    sq.sq_w4a4_gemm_decode(Qx[:0], sx[:0], Qt, sw, Y[:0])   # no tokens: nothing enqueued


def test_decode_path_captured_in_a_graph_replays_correctly(oracle):
    """The decode path a serving loop would record (sq_rotate_quantize_prepared, then
    sq_w4a4_gemm_decode on the tiled weights; nothing allocates, nothing but kernel launches):
    three replays on fresh inputs, with eager work and synchronizations in between, equal the
    eager two calls on the canonical weights bit for bit."""
    print("case graph capture of the decode path", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS["decode"]
    T, N = 8, 1100
    L = synth.layer(cfg, T)
    K = cfg.K
    Qw_h = synth.random_codes(N, K, 99)
    Qw, sw = dev(Qw_h), dev(np.random.default_rng(3).uniform(1e-3, 1e-2, N).astype(np.float32))
    Qt = run_tile_decode(Qw_h)
    R1, R2 = dev(L.R1), dev(L.R2)
    prepared = torch.empty((sq.sq_prepared_rotation_bytes(cfg.n1, cfg.n2),), dtype=torch.uint8, device="cuda")
    sq.sq_prepare_rotation(R1, R2, prepared)
    X = dev(L.X)
    Xin = torch.empty_like(X)
    Q = torch.empty((T, K // 2), dtype=torch.uint8, device="cuda")
    s = torch.empty((T,), dtype=torch.float32, device="cuda")
    Y = torch.empty((T, N), dtype=torch.float16, device="cuda")

    def step(stream):
        sq.sq_rotate_quantize_prepared(Xin, L.giv_i, L.giv_j, L.giv_theta, prepared, cfg.n1, cfg.n2, Q, s, stream=stream)
        sq.sq_w4a4_gemm_decode(Q, s, Qt, sw, Y, stream=stream)

    side = torch.cuda.Stream()
    Xin.copy_(X)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):                   # warm-up outside capture (one-time kernel attributes)
        step(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(side)
    for shift in (0, 3, 5):
        Xs = torch.roll(X, shift, 0).contiguous()
        Xin.copy_(Xs)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (Q.clone(), s.clone(), Y.clone())
        Qe, se, Ye = torch.empty_like(Q), torch.empty_like(s), torch.empty_like(Y)
        sq.sq_rotate_quantize(Xs, L.giv_i, L.giv_j, L.giv_theta, R1, R2, Qe, se)
        sq.sq_w4a4_gemm(Qe, se, Qw, sw, Ye)
        torch.cuda.synchronize()
        assert torch.equal(got[0], Qe) and torch.equal(got[1], se) and torch.equal(got[2], Ye), f"replay with shift {shift}"
