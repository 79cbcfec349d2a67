"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Element by element at sizes the oracle finishes in seconds; sampled rows,
sampled elements and exact checksums at the full benchmark sizes."""
import numpy as np
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

from paper_2511_22316_amd import synth
from parity_util import (Y_ROW_TOL, check_codes, check_rotation, codes_of, half_ulp_distance,
                         run_gemm, run_rotate_quantize)

pytestmark = pytest.mark.gpu


def _oracle_rq(oracle, L, X=None):
    X = L.X if X is None else X
    xr = oracle.rotate(X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Q, s = oracle.quantize_rows(xr)
    return xr, Q, s


# ------------------------------------------------------------------ rotate + quantize -----

@pytest.mark.parametrize("name,T", [("tiny", 16), ("attn_proj", 77), ("mlp_down", 40), ("decode", 8),
                                    ("large_prefill", 33)])
def test_rotate_quantize_elementwise(oracle, name, T):
    print(f"case rotate_quantize {name} T={T}", flush=True)
    L = synth.layer(synth.CONFIGS[name], T)
    Qg, sg, xg = run_rotate_quantize(L)
    xo, Qo, so = _oracle_rq(oracle, L)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)
    # the quantizer alone, decided in the kernel's precision: the oracle's fp32 quantizer fed
    # with the GPU's own rotated rows must give the GPU's codes (up to 1-ulp ties in x/s + 1/2)
    Qf, sf = oracle.quantize_rows(xg)
    assert np.array_equal(sf, sg)
    d = np.abs(codes_of(Qf) - codes_of(Qg))
    assert d.max() <= 1 and np.count_nonzero(d) <= 1e-5 * d.size + 1


def test_rotate_quantize_full_attn_proj(oracle):
    print("case rotate_quantize attn_proj full", flush=True)
    L = synth.layer(synth.CONFIGS["attn_proj"])
    Qg, sg, xg = run_rotate_quantize(L)
    xo, Qo, so = _oracle_rq(oracle, L)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)
    # without the debug output the codes must be the same bytes
    Qg2, sg2, _ = run_rotate_quantize(L, want_xrot=False)
    assert np.array_equal(Qg, Qg2) and np.array_equal(sg, sg2)


@pytest.mark.parametrize("name", ["mlp_down", "large_prefill"])
def test_rotate_quantize_full_size_sampled_rows(oracle, name):
    print(f"case rotate_quantize {name} full size, sampled rows", flush=True)
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg)
    rows = np.unique(np.concatenate([[0, 1, cfg.T - 1], np.random.default_rng(1).integers(0, cfg.T, 45)]))
    Qg, sg, xg = run_rotate_quantize(L, xrot_rows=rows)
    xo, Qo, so = _oracle_rq(oracle, L, L.X[rows])
    check_rotation(xg, xo)
    check_codes(Qg[rows], sg[rows], Qo, so)
    # the timed configuration (no debug output) writes the same codes and steps
    Qg2, sg2, _ = run_rotate_quantize(L, want_xrot=False)
    assert np.array_equal(Qg, Qg2) and np.array_equal(sg, sg2)
    # properties that hold for every row: full use of the range, |code| <= 7
    q = codes_of(Qg)
    assert np.all(np.max(np.abs(q), axis=1) == 7)


def test_rotate_quantize_edge_cases(oracle):
    print("case rotate_quantize edge cases", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS["tiny"]
    L = synth.layer(cfg)
    # an all-zero token, a token that is exactly representable after rotation by identity
    X = L.X.copy()
    X[3] = 0
    Qg, sg, xg = run_rotate_quantize(L, X)
    xo, Qo, so = _oracle_rq(oracle, L, X)
    assert sg[3] == 1.0 and np.all(Qg[3] == 0) and np.all(xg[3] == 0)
    check_rotation(np.delete(xg, 3, 0), np.delete(xo, 3, 0))
    check_codes(Qg, sg, Qo, so)
    # no Givens pairs at all
    L0 = synth.Layer(cfg, L.X, L.giv_i[:0], L.giv_j[:0], L.giv_theta[:0], L.R1, L.R2, L.R1_f64, L.R2_f64)
    Qg, sg, xg = run_rotate_quantize(L0)
    xo, Qo, so = _oracle_rq(oracle, L0)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)
    # T = 0 enqueues nothing and succeeds
    e = torch.empty((0, cfg.K), dtype=torch.float16, device="cuda")
    sq.sq_rotate_quantize(e, L.giv_i, L.giv_j, L.giv_theta, torch.from_numpy(L.R1).cuda(),
                          torch.from_numpy(L.R2).cuda(),
                          torch.empty((0, cfg.K // 2), dtype=torch.uint8, device="cuda"),
                          torch.empty((0,), dtype=torch.float32, device="cuda"))
    # a strided X (ldx > K) reads the right rows
    wide = torch.zeros((cfg.T, cfg.K + 64), dtype=torch.float16, device="cuda")
    wide[:, : cfg.K] = torch.from_numpy(L.X).cuda()
    Q = torch.empty((cfg.T, cfg.K // 2), dtype=torch.uint8, device="cuda")
    s = torch.empty((cfg.T,), dtype=torch.float32, device="cuda")
    sq.sq_rotate_quantize(wide[:, : cfg.K], L.giv_i, L.giv_j, L.giv_theta, torch.from_numpy(L.R1).cuda(),
                          torch.from_numpy(L.R2).cuda(), Q, s)
    torch.cuda.synchronize()
    Qref, sref, _ = run_rotate_quantize(L, want_xrot=False)
    assert np.array_equal(Q.cpu().numpy(), Qref) and np.array_equal(s.cpu().numpy(), sref)


@pytest.mark.parametrize("kind", ["chain_21", "star_16", "star_17", "disjoint_64", "repeat_pair", "two_trees_64",
                                  "many_q"])
@pytest.mark.parametrize("name", ["tiny", "attn_proj"])
def test_rotate_quantize_givens_list_shapes(oracle, name, kind):
    """Lists of different dependency structure: a chain (every pair waits for the one before), stars
    (one channel in every pair), 64 independent pairs, a pair repeated back to back, trees that
    use the longest list, and channels that fall on many different columns of the n1 x n2 view."""
    print(f"case rotate_quantize givens list {name} {kind}", flush=True)
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg, 12)
    K = cfg.K
    kinds = ["chain_21", "star_16", "star_17", "disjoint_64", "repeat_pair", "two_trees_64", "many_q"]
    g = np.random.default_rng(1000 * kinds.index(kind) + K)
    ch = g.permutation(K)
    if kind == "chain_21":          # 21 channels, every pair depends on the one before
        gi, gj = ch[:20], ch[1:21]
    elif kind == "star_16":         # 15 pairs through one channel
        gi, gj = np.full(15, ch[0]), ch[1:16]
    elif kind == "star_17":
        gi, gj = np.full(16, ch[0]), ch[1:17]
    elif kind == "disjoint_64":     # 64 pairs, 128 distinct channels: one level
        gi, gj = ch[:64], ch[64:128]
    elif kind == "repeat_pair":     # same two channels three times, then swapped
        gi, gj = np.array([ch[0], ch[0], ch[0], ch[1]]), np.array([ch[1], ch[1], ch[1], ch[0]])
    elif kind == "two_trees_64":    # two groups of 16 channels and a few small ones, 64 pairs in all
        a = [(ch[0], ch[1 + k % 15]) for k in range(30)] + [(ch[20], ch[21 + k % 15]) for k in range(30)]
        a += [(ch[40], ch[41]), (ch[42], ch[43]), (ch[41], ch[44]), (ch[43], ch[45])]
        gi, gj = np.array([x for x, _ in a]), np.array([y for _, y in a])
    else:                           # 32 pairs whose 64 channels sit in 64 different columns if n2 allows
        cols = g.permutation(cfg.n2)[: min(64, cfg.n2)]
        chans = np.array([g.integers(0, cfg.n1) * cfg.n2 + c for c in cols])
        gi, gj = chans[: len(chans) // 2], chans[len(chans) // 2: 2 * (len(chans) // 2)]
    gt = g.uniform(-3.1, 3.1, len(gi)).astype(np.float32)
    L2 = synth.Layer(cfg, L.X, gi.astype(np.int32), gj.astype(np.int32), gt, L.R1, L.R2, L.R1_f64, L.R2_f64)
    Qg, sg, xg = run_rotate_quantize(L2)
    xo, Qo, so = _oracle_rq(oracle, L2)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)


@pytest.mark.parametrize("name", ["decode", "mlp_down"])
def test_rotate_quantize_givens_list_touching_every_column(oracle, name):
    """64 pairs whose 128 channels fall on 128 different columns of the n1 x 128 view: the most
    columns a list can touch."""
    print(f"case rotate_quantize givens list wide {name}", flush=True)
    cfg = synth.CONFIGS[name]
    assert cfg.n2 == 128
    L = synth.layer(cfg, 10)
    g = np.random.default_rng(77 + cfg.n1)
    chans = np.array([g.integers(0, cfg.n1) * cfg.n2 + q for q in g.permutation(cfg.n2)])
    gi, gj = chans[:64].astype(np.int32), chans[64:].astype(np.int32)
    gt = g.uniform(-3.1, 3.1, 64).astype(np.float32)
    L2 = synth.Layer(cfg, L.X, gi, gj, gt, L.R1, L.R2, L.R1_f64, L.R2_f64)
    Qg, sg, xg = run_rotate_quantize(L2)
    xo, Qo, so = _oracle_rq(oracle, L2)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)


@pytest.mark.parametrize("n1,n2,P", [(32, 32, 8), (32, 64, 16), (80, 64, 24),      # matrix-core kernel
                                     (80, 64, 6), (80, 64, 0), (86, 128, 0),        # ... with R1 shared in LDS
                                     (128, 64, 32), (108, 128, 24), (112, 128, 64), (128, 128, 48),
                                     (24, 40, 6), (12, 8, 3), (128, 16, 10)])       # generic kernel
def test_rotate_quantize_other_factor_shapes(oracle, n1, n2, P):
    """Factor pairs beyond the five benchmark layers: the remaining instantiations of the
    matrix-core kernel and shapes only the generic kernel takes."""
    print(f"case rotate_quantize shape {n1}x{n2}", flush=True)
    cfg = synth.LayerConfig(f"shape_{n1}x{n2}", 37, n1, n2, 64, P, "normal", 3, 300.0, 0.01, 20.0, 0.02, 4242 + n1 * n2)
    L = synth.layer(cfg)
    Qg, sg, xg = run_rotate_quantize(L)
    xo, Qo, so = _oracle_rq(oracle, L)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)


@pytest.mark.parametrize("n1,n2,wide_list", [(128, 64, False), (112, 128, True)])
def test_rotate_quantize_four_row_blocks_many_tokens(oracle, n1, n2, wide_list):
    """Shapes with four 32-row blocks (8192 = 128 x 64 is the split Alg. 1 picks; 14336 = 112 x 128)
    with enough tokens that every workgroup walks its ring several times; sampled rows against
    the oracle.  The second case carries a list whose channels fall on 128 different columns."""
    print(f"case rotate_quantize shape {n1}x{n2} many tokens", flush=True)
    T = 1700 if n2 == 64 else 900
    cfg = synth.LayerConfig(f"shape_{n1}x{n2}_long", T, n1, n2, 64, 32, "normal", 3, 300.0, 0.01, 20.0, 0.02, 99 + n1)
    L = synth.layer(cfg)
    if wide_list:
        g = np.random.default_rng(5 + n1)
        chans = np.array([g.integers(0, n1) * n2 + q for q in g.permutation(n2)])
        L = synth.Layer(cfg, L.X, chans[:64].astype(np.int32), chans[64:].astype(np.int32),
                        g.uniform(-3.1, 3.1, 64).astype(np.float32), L.R1, L.R2, L.R1_f64, L.R2_f64)
    Qg, sg, xg = run_rotate_quantize(L)
    rows = np.unique(np.concatenate([[0, 1, T - 2, T - 1], np.random.default_rng(2).integers(0, T, 60)]))
    xo, Qo, so = _oracle_rq(oracle, L, L.X[rows])
    check_rotation(xg[rows], xo)
    check_codes(Qg[rows], sg[rows], Qo, so)
    assert np.all(np.max(np.abs(codes_of(Qg)), axis=1) == 7)


@pytest.mark.parametrize("T,with_list", [(5000, True), (5000, False), (4097, True), (3100, True)])
def test_rotate_quantize_64x64_many_tokens(oracle, T, with_list):
    """From 4096 tokens on, the 64 x 64 shape runs with a ring of two tiles and three workgroups per
    CU: 5000 tokens (every workgroup walks its ring several times, the last pass is ragged) and
    4097 (the last pair of token slots is half empty), sampled rows against the oracle, with the
    layer's Givens list and without one.  At 3100 tokens only the entry point with prepared
    operands takes that variant, so the two entry points' equal results there come from two
    different launch shapes."""
    print(f"case rotate_quantize attn_proj T={T} list={with_list}", flush=True)
    cfg = synth.CONFIGS["attn_proj"]
    L = synth.layer(cfg, T)
    if not with_list:
        e = np.zeros(0, np.int32)
        L = synth.Layer(cfg, L.X, e, e, np.zeros(0, np.float32), L.R1, L.R2, L.R1_f64, L.R2_f64)
    Qg, sg, xg = run_rotate_quantize(L)
    rows = np.unique(np.concatenate([[0, 1, 767, 768, 1535, 1536, T - 2, T - 1],
                                     np.random.default_rng(8).integers(0, T, 80)]))
    xo, Qo, so = _oracle_rq(oracle, L, L.X[rows])
    check_rotation(xg[rows], xo)
    check_codes(Qg[rows], sg[rows], Qo, so)
    assert np.all(np.max(np.abs(codes_of(Qg)), axis=1) == 7)
    Qg2, sg2, _ = run_rotate_quantize(L, want_xrot=False)
    assert np.array_equal(Qg, Qg2) and np.array_equal(sg, sg2)


def test_rotate_quantize_generic_kernel_on_benchmark_shape(oracle):
    """The plain-FMA kernel, forced on a shape the matrix-core kernel normally takes, must agree
    with the oracle as well (it is the fallback for every shape without an instantiation)."""
    print("case rotate_quantize plain kernel forced", flush=True)
    import paper_2511_22316_amd as sq
    L = synth.layer(synth.CONFIGS["attn_proj"], 20)
    sq.sq_debug_set_option(sq.binding.SQ_DEBUG_ROTQ_PLAIN_KERNEL, 1)
    try:
        Qg, sg, xg = run_rotate_quantize(L)
    finally:
        sq.sq_debug_set_option(sq.binding.SQ_DEBUG_ROTQ_PLAIN_KERNEL, 0)
    xo, Qo, so = _oracle_rq(oracle, L)
    check_rotation(xg, xo)
    check_codes(Qg, sg, Qo, so)
    # the two kernels round their sums differently, so the forced run is not the normal one
    _, _, xm = run_rotate_quantize(L)
    assert not np.array_equal(xm, xg)
    check_rotation(xm, xo)


def test_rotate_quantize_identity_rotation_is_exact(oracle):
    """R1 = I, R2 = I, no Givens: the rotated row is the fp16 input itself, bit for bit."""
    print("case rotate_quantize identity", flush=True)
    cfg = synth.CONFIGS["tiny"]
    L = synth.layer(cfg)
    Li = synth.Layer(cfg, L.X, L.giv_i[:0], L.giv_j[:0], L.giv_theta[:0],
                     np.eye(cfg.n1, dtype=np.float16), np.eye(cfg.n2, dtype=np.float16), None, None)
    Qg, sg, xg = run_rotate_quantize(Li)
    assert np.array_equal(xg, L.X.astype(np.float32))
    Qo, so = oracle.quantize_rows(L.X.astype(np.float64))
    check_codes(Qg, sg, Qo, so)


def _tie_rows(n_rows, K, delta):
    """Rows whose largest |entry| is 7 delta (so the step is exactly delta) and whose other
    entries are k delta and (k + 1/2) delta: every second one an exact rounding tie."""
    halves = np.arange(-13, 14, dtype=np.float64) / 2.0            # -6.5, -6, ..., 6, 6.5
    X = np.empty((n_rows, K), np.float64)
    for r in range(n_rows):
        X[r] = np.roll(np.resize(halves, K), 5 * r)
        X[r, (11 * r + 3) % K] = 7.0 if r % 2 == 0 else -7.0
    return (X * delta).astype(np.float16)


@pytest.mark.parametrize("n1,n2", [(16, 32), (64, 64), (64, 128), (86, 128), (12, 8)])
@pytest.mark.parametrize("delta", [1.0, 2.0, 0.25])
def test_rounding_ties_go_up(oracle, n1, n2, delta):
    """The quantizer of Sec. 3.2 is floor(z / Delta + 1/2): exact ties round UP (0.5 -> 1,
    -0.5 -> 0, -2.5 -> -2).  With R1 = R2 = I and no Givens list the rotated row is the input,
    the step is exactly Delta, every quotient is exact in fp32, and the codes must EQUAL the
    oracle's: no flip allowance.  Matrix-core shapes and a shape only the plain kernel takes."""
    print(f"case rounding ties {n1}x{n2} delta={delta}", flush=True)
    K = n1 * n2
    X = _tie_rows(9, K, delta)
    cfg = synth.LayerConfig(f"ties_{n1}x{n2}", 9, n1, n2, 8, 0, "normal", 0, 1.0, 0.0, 1.0, 0.02, 1)
    e = np.zeros(0, np.int32)
    Li = synth.Layer(cfg, X, e, e, np.zeros(0, np.float32), np.eye(n1, dtype=np.float16),
                     np.eye(n2, dtype=np.float16), None, None)
    Qg, sg, xg = run_rotate_quantize(Li)
    assert np.array_equal(xg, X.astype(np.float32))
    Qo, so = oracle.quantize_rows(X.astype(np.float64))
    assert np.all(so == np.float32(delta)) and np.array_equal(sg, so)
    assert np.array_equal(Qg, Qo), "a tie was not rounded up"
    # and the rule itself, from the definition, on the GPU's codes
    want = np.clip(np.floor(X.astype(np.float64) / delta + 0.5), -8, 7).astype(np.int16)
    assert np.array_equal(codes_of(Qg), want)
    assert np.count_nonzero(X.astype(np.float64) / delta % 1 == 0.5) > K      # the ties are there


# ------------------------------------------------------------------------------ GEMM ------

@pytest.mark.parametrize("T,K,N", [(1, 32, 1), (16, 512, 512), (77, 96, 300), (130, 288, 257),
                                   (8, 1024, 520), (300, 2048, 130),
                                   # at most 32 tokens: the decode-shaped kernel in its three launch
                                   # shapes, one K slice only / ragged channel tails / T = 32
                                   (1, 256, 33), (32, 768, 8200), (16, 512, 10300), (31, 512, 24600), (33, 512, 300),
                                   # ... with the token rows held in LDS over several 1 KB pieces
                                   # (15 rows of 4 KB are the most that fit) and without (too many rows)
                                   (8, 8192, 25000), (15, 8192, 700), (5, 2304, 12000), (16, 8192, 700), (32, 8192, 300),
                                   (20, 4096, 10300),
                                   # 33..64 tokens: the same kernel with two token blocks (few
                                   # channels) or 64x64 tiles (many); 65..128 tokens: 64x64 tiles
                                   (64, 768, 16500), (48, 512, 300), (40, 512, 30000), (20, 256, 25000),
                                   (100, 512, 260), (128, 256, 64),
                                   # a few hundred tokens: 64x64, 64x128 and 128x128 tiles
                                   (129, 512, 520), (400, 768, 1000), (512, 512, 4096), (300, 512, 8200),
                                   # K % 512 == 0 and at most 256 small tiles: two K groups per
                                   # workgroup (64x64 and 64x128 tiles), next to shapes just outside
                                   (64, 1024, 8200), (200, 1536, 4100), (50, 512, 40000), (64, 512, 16385)])
def test_gemm_random_codes_bit_exact(oracle, T, K, N):
    print(f"case gemm random codes T={T} K={K} N={N}", flush=True)
    g = np.random.default_rng(T * 7 + K + N)
    Qx = synth.random_codes(T, K, 100 + T)        # all 16 codes, -8 included
    Qw = synth.random_codes(N, K, 200 + N)
    sx = g.uniform(0.05, 4.0, T).astype(np.float32)
    sw = g.uniform(1e-4, 5e-3, N).astype(np.float32)
    Yg, accg = run_gemm(Qx, sx, Qw, sw)
    Yo, acco = oracle.gemm(Qx, sx, Qw, sw)
    assert np.array_equal(accg, acco)
    assert half_ulp_distance(Yg, Yo).max() <= 1
    # extreme codes: every product is (-8)(-8)
    Qm = np.full((T, K // 2), 0x88, np.uint8)
    Qn = np.full((N, K // 2), 0x88, np.uint8)
    _, accm = run_gemm(Qm, sx, Qn, sw)
    assert np.all(accm == 64 * K)


@pytest.mark.parametrize("case", [0, 1, 2, 3, 4, 5, 6, 10, 11, 16, 17])
@pytest.mark.parametrize("T,K,N", [(300, 512, 520), (130, 768, 257), (70, 256, 300)])      # the last: a single K tile
def test_gemm_every_tile_launch_shape(oracle, case, T, K, N):
    """Every launch shape of the tile kernel (tile sizes, waves per workgroup, the form with
    separate loading waves), forced through the debug option onto shapes with ragged token and
    channel tails: int32 accumulators bit-exact, Y within one fp16 ulp."""
    print(f"case gemm forced launch shape {case} T={T} K={K} N={N}", flush=True)
    import paper_2511_22316_amd as sq
    g = np.random.default_rng(case + T + K + N)
    Qx = synth.random_codes(T, K, 500 + T)
    Qw = synth.random_codes(N, K, 600 + N)
    sx = g.uniform(0.05, 4.0, T).astype(np.float32)
    sw = g.uniform(1e-4, 5e-3, N).astype(np.float32)
    Yo, acco = oracle.gemm(Qx, sx, Qw, sw)
    sq.sq_debug_set_option(sq.binding.SQ_DEBUG_GEMM_LAUNCH_SHAPE, case + 1)
    try:
        Yg, accg = run_gemm(Qx, sx, Qw, sw)
    finally:
        sq.sq_debug_set_option(sq.binding.SQ_DEBUG_GEMM_LAUNCH_SHAPE, 0)
    assert np.array_equal(accg, acco)
    assert half_ulp_distance(Yg, Yo).max() <= 1


def test_gemm_seeded_random_shapes_bit_exact(oracle):
    """Thirty shapes drawn from a seed (T up to 700, K a multiple of 32 up to 2304, N up to 3000, a
    third of them with at most 64 tokens): whatever kernel and launch shape the dispatcher picks,
    the int32 accumulators are the oracle's and Y is within one fp16 ulp."""
    g = np.random.default_rng(20251122)
    for case in range(30):
        T = int(g.integers(1, 65)) if case % 3 == 0 else int(g.integers(65, 700))
        K = 32 * int(g.integers(1, 73))
        N = int(g.integers(1, 3000))
        print(f"case gemm seeded shape {case}: T={T} K={K} N={N}", flush=True)
        Qx = synth.random_codes(T, K, 700 + case)
        Qw = synth.random_codes(N, K, 800 + case)
        sx = g.uniform(0.05, 4.0, T).astype(np.float32)
        sw = g.uniform(1e-4, 5e-3, N).astype(np.float32)
        Yg, accg = run_gemm(Qx, sx, Qw, sw)
        Yo, acco = oracle.gemm(Qx, sx, Qw, sw)
        assert np.array_equal(accg, acco), f"accumulators differ at T={T} K={K} N={N}"
        assert half_ulp_distance(Yg, Yo).max() <= 1


def test_gemm_strided_output_and_empty(oracle):
    print("case gemm strided output / empty", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    T, K, N = 40, 256, 72
    Qx, Qw = synth.random_codes(T, K, 1), synth.random_codes(N, K, 2)
    sx = np.full(T, 0.5, np.float32)
    sw = np.full(N, 0.25, np.float32)
    Ywide = torch.full((T, N + 10), -1.0, dtype=torch.float16, device="cuda")
    sq.sq_w4a4_gemm(torch.from_numpy(Qx).cuda(), torch.from_numpy(sx).cuda(), torch.from_numpy(Qw).cuda(),
                    torch.from_numpy(sw).cuda(), Ywide[:, :N])
    torch.cuda.synchronize()
    Yo, _ = oracle.gemm(Qx, sx, Qw, sw)
    got = Ywide.cpu().numpy()
    assert np.array_equal(got[:, :N], Yo) and np.all(got[:, N:] == -1.0)
    sq.sq_w4a4_gemm(torch.empty((0, K // 2), dtype=torch.uint8, device="cuda"),
                    torch.empty((0,), dtype=torch.float32, device="cuda"),
                    torch.from_numpy(Qw).cuda(), torch.from_numpy(sw).cuda(),
                    torch.empty((0, N), dtype=torch.float16, device="cuda"))


# --------------------------------------------------------------- the whole layer ----------

def _gpu_weights(L, Wt):
    """Offline weight path on the GPU: the rows of W^T take the same transform and the same
    quantizer as token rows (Sec. 4.2, Flat(W~_R) = W^T R)."""
    Q, s, _ = run_rotate_quantize(L, Wt, want_xrot=False)
    return Q, s


@pytest.mark.parametrize("name", ["tiny", "decode_small"])
def test_layer_end_to_end(oracle, name):
    print(f"case layer end to end {name}", flush=True)
    if name == "tiny":
        cfg, N = synth.CONFIGS["tiny"], 512
    else:
        cfg, N = synth.CONFIGS["decode"], 300
    L = synth.layer(cfg)
    Wt = synth.weights_t(cfg, N)
    # oracle pipeline
    xo, Qxo, sxo = _oracle_rq(oracle, L)
    Qwo, swo = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Yo, acco = oracle.gemm(Qxo, sxo, Qwo, swo)
    # GPU GEMM on the oracle's codes: exact accumulators, Y within one fp16 ulp
    Yg1, accg1 = run_gemm(Qxo, sxo, Qwo, swo)
    assert np.array_equal(accg1, acco) and half_ulp_distance(Yg1, Yo).max() <= 1
    # GPU pipeline end to end (its own codes on both sides)
    Qxg, sxg, _ = run_rotate_quantize(L, want_xrot=False)
    Qwg, swg = _gpu_weights(L, Wt)
    check_codes(Qwg, swg, Qwo, swo)
    Yg, _ = run_gemm(Qxg, sxg, Qwg, swg)
    d = Yg.astype(np.float64) - Yo.astype(np.float64)
    rel = np.linalg.norm(d, axis=1) / np.linalg.norm(Yo.astype(np.float64), axis=1)
    assert rel.max() <= Y_ROW_TOL, f"fp16 Y: worst row error {rel.max():.3e}"


@pytest.mark.parametrize("name,n_rows", [("attn_proj", 0), ("mlp_down", 72), ("large_prefill", 64)])
def test_layer_full_size_y_against_oracle_pipeline(oracle, name, n_rows):
    """The final fp16 Y of the GPU pipeline (its own codes on both operands, full benchmark size,
    the launch configuration the benchmark times) against the Y of the oracle pipeline (its own
    codes on both operands): per token row ||dY|| / ||Y|| <= 1e-2.  attn_proj on every token;
    the larger layers on sampled token rows times all N output channels."""
    print(f"case layer full size Y vs oracle pipeline {name}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg)
    T, K, N = cfg.T, cfg.K, cfg.N
    rows = (np.arange(T) if n_rows == 0 else
            np.unique(np.concatenate([[0, T - 1], np.random.default_rng(17).integers(0, T, n_rows)])))
    dR1, dR2, dX = torch.from_numpy(L.R1).cuda(), torch.from_numpy(L.R2).cuda(), torch.from_numpy(L.X).cuda()
    Qw_d = torch.empty((N, K // 2), dtype=torch.uint8, device="cuda")
    sw_d = torch.empty((N,), dtype=torch.float32, device="cuda")
    Qwo = np.empty((N, K // 2), np.uint8)
    swo = np.empty((N,), np.float32)
    step = 4096
    for lo in range(0, N, step):                      # weights drawn and prepared in slabs, on both sides
        hi = min(N, lo + step)
        Wt = synth.weight_rows_t(cfg, np.arange(lo, hi))
        sq.sq_rotate_quantize(torch.from_numpy(Wt).cuda(), L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, Qw_d[lo:hi], sw_d[lo:hi])
        Qwo[lo:hi], swo[lo:hi] = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
        print(f"  weights {hi}/{N}", flush=True)
    Qx_d = torch.empty((T, K // 2), dtype=torch.uint8, device="cuda")
    sx_d = torch.empty((T,), dtype=torch.float32, device="cuda")
    Y_d = torch.empty((T, N), dtype=torch.float16, device="cuda")
    sq.sq_rotate_quantize(dX, L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, Qx_d, sx_d)
    sq.sq_w4a4_gemm(Qx_d, sx_d, Qw_d, sw_d, Y_d)
    torch.cuda.synchronize()
    Yg = Y_d[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    _, Qxo, sxo = _oracle_rq(oracle, L, L.X[rows])
    Yo, _ = oracle.gemm(Qxo, sxo, Qwo, swo)
    Yo = Yo.astype(np.float64)
    rel = np.linalg.norm(Yg - Yo, axis=1) / np.linalg.norm(Yo, axis=1)
    print(f"  worst row error {rel.max():.3e} over {len(rows)} rows", flush=True)
    assert rel.max() <= Y_ROW_TOL, f"fp16 Y: worst row error {rel.max():.3e}"


@pytest.mark.parametrize("name", ["attn_proj", "mlp_down", "decode", "large_prefill"])
def test_gemm_full_size_checksums_and_samples(oracle, name):
    """Full benchmark shapes, the launch configuration the benchmark times: exact int64 checksum
    invariants over every accumulator, sampled accumulators from the oracle, and Y recomputed
    from the accumulators on sampled rows."""
    print(f"case gemm full size {name}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg)
    Qx, sx, _ = run_rotate_quantize(L, want_xrot=False)
    T, K, N = cfg.T, cfg.K, cfg.N
    dR1, dR2 = torch.from_numpy(L.R1).cuda(), torch.from_numpy(L.R2).cuda()
    Qw_d = torch.empty((N, K // 2), dtype=torch.uint8, device="cuda")
    sw_d = torch.empty((N,), dtype=torch.float32, device="cuda")
    step = 4096
    for lo in range(0, N, step):                      # weights drawn and prepared in slabs
        hi = min(N, lo + step)
        Wt = torch.from_numpy(synth.weight_rows_t(cfg, np.arange(lo, hi))).cuda()
        sq.sq_rotate_quantize(Wt, L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, Qw_d[lo:hi], sw_d[lo:hi])
    torch.cuda.synchronize()
    Qw, sw = Qw_d.cpu().numpy(), sw_d.cpu().numpy()
    Y_d = torch.empty((T, N), dtype=torch.float16, device="cuda")
    acc_d = torch.empty((T, N), dtype=torch.int32, device="cuda")
    sq.sq_w4a4_gemm(torch.from_numpy(Qx).cuda(), torch.from_numpy(sx).cuda(), Qw_d, sw_d, Y_d, acc_d)
    torch.cuda.synchronize()
    col_sum = acc_d.sum(dim=0, dtype=torch.int64).cpu().numpy()
    row_sum = acc_d.sum(dim=1, dtype=torch.int64).cpu().numpy()
    # sums of codes are small integers: float64 matrix products are exact here
    cx = codes_of(Qx).astype(np.float64)
    cw = codes_of(Qw).astype(np.float64)
    assert np.array_equal(col_sum, (cx.sum(axis=0) @ cw.T).astype(np.int64))
    assert np.array_equal(row_sum, (cx @ cw.sum(axis=0)).astype(np.int64))
    g = np.random.default_rng(5)
    ts = np.concatenate([[0, T - 1], g.integers(0, T, 30)])
    ns = np.concatenate([[0, N - 1], g.integers(0, N, 30)])
    acc_s = acc_d[torch.from_numpy(ts).cuda()][:, torch.from_numpy(ns).cuda()].cpu().numpy()
    for a, t in enumerate(ts):
        for b, n in enumerate(ns):
            assert acc_s[a, b] == oracle.gemm_acc_at(Qx, Qw, int(t), int(n))
    rows = torch.from_numpy(ts).cuda()
    acc_rows = acc_d[rows].cpu().numpy().astype(np.float64)
    want = (acc_rows * sx[ts, None].astype(np.float64) * sw[None, :].astype(np.float64)).astype(np.float16)
    assert half_ulp_distance(Y_d[rows].cpu().numpy(), want).max() <= 1
    # the run without the debug output writes the same Y
    Y2 = torch.empty_like(Y_d)
    sq.sq_w4a4_gemm(torch.from_numpy(Qx).cuda(), torch.from_numpy(sx).cuda(), Qw_d, sw_d, Y2)
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y_d)
    # weight codes of sampled output channels against the oracle's offline path
    Qwo, swo = oracle.prepare_weights(synth.weight_rows_t(cfg, ns), L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    check_codes(Qw[ns], sw[ns], Qwo, swo)


# ------------------------------------------------------------------ offline weight path -----

@pytest.mark.parametrize("name,N", [("tiny", 512), ("tiny", 130), ("attn_proj", 200)])
def test_prepare_weights_matches_oracle(oracle, name, N):
    """sq_prepare_weights on W [K, N] against the oracle's weight path on the rows of W^T; then
    the codes it wrote feed sq_w4a4_gemm and the accumulators are the oracle's, bit for bit."""
    print(f"case prepare_weights {name} N={N}", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg, 16)
    Wt = synth.weights_t(cfg, N)                          # [N, K] fp16
    W = torch.from_numpy(np.ascontiguousarray(Wt.T)).cuda()    # [K, N]
    wide = torch.zeros((cfg.K, N + 24), dtype=torch.float16, device="cuda")   # strided source
    wide[:, :N] = W
    ws = torch.empty((N * cfg.K,), dtype=torch.float16, device="cuda")
    Qw = torch.empty((N, cfg.K // 2), dtype=torch.uint8, device="cuda")
    sw = torch.empty((N,), dtype=torch.float32, device="cuda")
    R1, R2 = torch.from_numpy(L.R1).cuda(), torch.from_numpy(L.R2).cuda()
    sq.sq_prepare_weights(wide[:, :N], L.giv_i, L.giv_j, L.giv_theta, R1, R2, ws, Qw, sw)
    torch.cuda.synchronize()
    assert np.array_equal(ws.cpu().numpy().reshape(N, cfg.K), Wt)        # the transpose is exact
    Qo, so = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    check_codes(Qw.cpu().numpy(), sw.cpu().numpy(), Qo, so)
    # same bytes as the row kernel applied to W^T directly
    Q2 = torch.empty_like(Qw)
    s2 = torch.empty_like(sw)
    sq.sq_rotate_quantize(torch.from_numpy(Wt).cuda(), L.giv_i, L.giv_j, L.giv_theta, R1, R2, Q2, s2)
    torch.cuda.synchronize()
    assert torch.equal(Q2, Qw) and torch.equal(s2, sw)
    # the prepared weights drive the GEMM
    Qx, sx, _ = run_rotate_quantize(L, want_xrot=False)
    Yg, accg = run_gemm(Qx, sx, Qw.cpu().numpy(), sw.cpu().numpy())
    _, acco = oracle.gemm(Qx, sx, Qw.cpu().numpy(), sw.cpu().numpy())
    assert np.array_equal(accg, acco)


# ------------------------------------------------------------------ streams -----

def test_layer_on_a_side_stream_matches_default_stream(oracle):
    """Both calls enqueue on the stream they are given and nowhere else: a layer run on a side
    stream, behind a long fill of its inputs on that stream, equals the run on the default one."""
    print("case side stream", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS["attn_proj"]
    L = synth.layer(cfg, 300)
    N = 384
    Wt = synth.weights_t(cfg, N)
    Qw_h, sw_h = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    dev = "cuda"
    R1, R2 = torch.from_numpy(L.R1).to(dev), torch.from_numpy(L.R2).to(dev)
    Qw, sw = torch.from_numpy(Qw_h).to(dev), torch.from_numpy(sw_h).to(dev)
    Xh = torch.from_numpy(L.X).pin_memory()

    def run(stream):
        X = torch.empty((300, cfg.K), dtype=torch.float16, device=dev)
        Q = torch.empty((300, cfg.K // 2), dtype=torch.uint8, device=dev)
        s = torch.empty((300,), dtype=torch.float32, device=dev)
        Y = torch.empty((300, N), dtype=torch.float16, device=dev)
        with torch.cuda.stream(stream):
            X.copy_(Xh, non_blocking=True)          # the kernels must wait for this copy: same stream
            sq.sq_rotate_quantize(X, L.giv_i, L.giv_j, L.giv_theta, R1, R2, Q, s, stream=stream)
            sq.sq_w4a4_gemm(Q, s, Qw, sw, Y, stream=stream)
        stream.synchronize()
        return Q.cpu().numpy(), s.cpu().numpy(), Y.cpu().numpy()

    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    Q1, s1, Y1 = run(side)
    Q0, s0, Y0 = run(torch.cuda.current_stream())
    assert np.array_equal(Q0, Q1) and np.array_equal(s0, s1) and np.array_equal(Y0, Y1)
    xo, Qo, so = _oracle_rq(oracle, L)
    check_codes(Q1, s1, Qo, so)


def test_layer_captured_in_a_graph_replays_correctly(oracle):
    """Both calls can be recorded into a HIP graph (they allocate nothing and only launch
    kernels): three replays, each on fresh contents of the static input buffer and with eager
    work and a synchronization in between, equal the eager results bit for bit."""
    print("case graph capture", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS["attn_proj"]
    T, N = 260, 512
    L = synth.layer(cfg, T)
    Wt = synth.weights_t(cfg, N)
    dev = "cuda"
    R1, R2 = torch.from_numpy(L.R1).to(dev), torch.from_numpy(L.R2).to(dev)
    Qw = torch.empty((N, cfg.K // 2), dtype=torch.uint8, device=dev)
    sw = torch.empty((N,), dtype=torch.float32, device=dev)
    sq.sq_rotate_quantize(torch.from_numpy(Wt).to(dev), L.giv_i, L.giv_j, L.giv_theta, R1, R2, Qw, sw)
    X = torch.from_numpy(L.X).to(dev)
    Xin = torch.empty_like(X)                       # static buffers of the graph
    Q = torch.empty((T, cfg.K // 2), dtype=torch.uint8, device=dev)
    s = torch.empty((T,), dtype=torch.float32, device=dev)
    Y = torch.empty((T, N), dtype=torch.float16, device=dev)

    def layer(stream):
        sq.sq_rotate_quantize(Xin, L.giv_i, L.giv_j, L.giv_theta, R1, R2, Q, s, stream=stream)
        sq.sq_w4a4_gemm(Q, s, Qw, sw, Y, stream=stream)

    side = torch.cuda.Stream()
    Xin.copy_(X)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):                   # warm-up outside capture (one-time kernel attributes)
        layer(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer(side)
    for shift in (0, 7, 101):
        Xs = torch.roll(X, shift, 0).contiguous()
        Xin.copy_(Xs)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (Q.clone(), s.clone(), Y.clone())
        Qe, se, Ye = torch.empty_like(Q), torch.empty_like(s), torch.empty_like(Y)   # eager, other buffers
        sq.sq_rotate_quantize(Xs, L.giv_i, L.giv_j, L.giv_theta, R1, R2, Qe, se)
        sq.sq_w4a4_gemm(Qe, se, Qw, sw, Ye)
        torch.cuda.synchronize()
        assert torch.equal(got[0], Qe) and torch.equal(got[1], se) and torch.equal(got[2], Ye), f"replay with shift {shift}"
