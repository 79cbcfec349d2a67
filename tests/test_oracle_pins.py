"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these compares the oracle with itself: each expected value is a closed form printed in
the paper, an explicit dense matrix product done by numpy, a brute force, an IEEE table, or a
hand-worked case.  CPU only.
"""
import math

import numpy as np
import pytest

from paper_2511_22316_amd import synth


# ------------------------------------------------------------------ fp16 ------------------

def test_half_decode_matches_ieee_table(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))
    assert np.array_equal(np.signbit(got[finite]), np.signbit(want[finite]))


def test_half_encode_round_nearest_even(oracle):
    g = np.random.default_rng(7)
    xs = np.concatenate([
        g.standard_normal(20000) * 10.0 ** g.uniform(-9, 5, 20000),
        # exact midpoints between neighbouring halfs, normal and subnormal: ties go to even
        np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 65504.0 + 16.0,
                  65504.0 + 15.999, 65520.0, 2.0 ** -14 - 2.0 ** -25, 0.0, -0.0, 1e-9, -1e-9, 7e4, -7e4]),
    ])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------- Sec. 4.1: Givens rotation, Lemma 1 ------

def _explicit_givens(n, i, j, theta):
    """n x n matrix of Sec. 4.1 / Lemma 1: identity except the 2x2 block
    [[cos, -sin], [sin, cos]] on rows and columns (i, j)."""
    G = np.eye(n)
    G[i, i] = math.cos(theta)
    G[i, j] = -math.sin(theta)
    G[j, i] = math.sin(theta)
    G[j, j] = math.cos(theta)
    return G


@pytest.mark.parametrize("n,i,j", [(2, 0, 1), (2, 1, 0), (7, 5, 2), (7, 0, 6)])
def test_givens_apply_is_row_vector_times_explicit_matrix(oracle, n, i, j):
    g = np.random.default_rng(n * 100 + i * 10 + j)
    for theta in [0.3, -1.1, 2.9, math.pi / 2]:
        x = g.standard_normal(n)
        G = _explicit_givens(n, i, j, theta)
        assert np.allclose(G.T @ G, np.eye(n), atol=1e-15)
        np.testing.assert_allclose(oracle.givens_apply(x, i, j, theta), x @ G, rtol=0, atol=1e-15)


def test_lemma1_closed_form_all_quadrants(oracle):
    # Lemma 1: V G(theta*) = (r/sqrt2, r/sqrt2) for theta* = atan2(b, a) - pi/4
    cases = [(3.0, 4.0), (-3.0, 4.0), (-3.0, -4.0), (3.0, -4.0), (0.0, 2.0), (2.0, 0.0),
             (-2.0, 0.0), (0.0, -2.0), (1e3, 1e-3), (-1e-3, 1e3)]
    for a, b in cases:
        th = oracle.art_angle(a, b)
        out = oracle.givens_apply(np.array([a, b]), 0, 1, th)
        r = math.hypot(a, b)
        np.testing.assert_allclose(out, [r / math.sqrt(2)] * 2, rtol=1e-14)
    # r = 0 is the trivial case of the proof
    out = oracle.givens_apply(np.zeros(2), 0, 1, oracle.art_angle(0.0, 0.0))
    assert np.array_equal(out, np.zeros(2))


def test_lemma1_angle_is_the_brute_force_minimiser(oracle):
    g = np.random.default_rng(11)
    grid = np.linspace(0.0, 2 * math.pi, 100001)
    for _ in range(6):
        a, b = g.standard_normal(2) * 10.0 ** g.uniform(-2, 3)
        r = math.hypot(a, b)
        # brute force of min over theta of ||(a,b) G(theta)||_inf using the explicit 2x2 matrix
        c, s = np.cos(grid), np.sin(grid)
        linf = np.maximum(np.abs(a * c + b * s), np.abs(b * c - a * s))
        assert linf.min() >= r / math.sqrt(2) * (1 - 1e-12)
        assert linf.min() <= r / math.sqrt(2) * (1 + 1e-4)
        th = oracle.art_angle(a, b)
        out = oracle.givens_apply(np.array([a, b]), 0, 1, th)
        assert abs(np.max(np.abs(out)) - r / math.sqrt(2)) <= 1e-13 * r
        # the grid minimiser is theta* up to the pi/2 symmetry of the infinity norm
        d = (grid[np.argmin(linf)] - th) % (math.pi / 2)
        assert min(d, math.pi / 2 - d) < 1e-4


# ------------------------------------------------------- Eq. 18: Kronecker identity --------

@pytest.mark.parametrize("n1,n2", [(2, 2), (3, 5), (5, 3), (8, 8), (4, 7), (1, 6), (6, 1)])
def test_kron_apply_equals_explicit_dense_kron(oracle, n1, n2):
    g = np.random.default_rng(n1 * 31 + n2)
    # general (non-orthogonal, non-symmetric) factors: a transposed operand cannot hide
    R1 = g.standard_normal((n1, n1))
    R2 = g.standard_normal((n2, n2))
    v = g.standard_normal(n1 * n2)
    want = v @ np.kron(R1, R2)
    np.testing.assert_allclose(oracle.kron_apply(v, R1, R2), want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.kron_apply_dense(v, R1, R2), want, rtol=1e-12, atol=1e-12)
    # and the matrix form of Eq. 18 itself, done by numpy
    np.testing.assert_allclose(oracle.kron_apply(v, R1, R2),
                               (R1.T @ v.reshape(n1, n2) @ R2).reshape(-1), rtol=1e-12, atol=1e-12)


def test_mode_product_identities(oracle):
    # Sec. 4.2: Flat(X~ x2 R1^T x3 R2^T) = X R with the paper's mode-product convention
    g = np.random.default_rng(5)
    T, n1, n2 = 4, 3, 4
    R1, R2 = g.standard_normal((n1, n1)), g.standard_normal((n2, n2))
    X = g.standard_normal((T, n1 * n2))
    Xt = X.reshape(T, n1, n2)
    # (A x2 M)[i,p,j] = sum_q A[i,q,j] M[p,q];  (A x3 N)[i,p,l] = sum_q A[i,p,q] N[l,q]
    m2 = np.einsum("iqj,pq->ipj", Xt, R1.T)
    m3 = np.einsum("ipq,lq->ipl", m2, R2.T)
    want = m3.reshape(T, -1)
    np.testing.assert_allclose(want, X @ np.kron(R1, R2), rtol=1e-12, atol=1e-12)
    got = np.stack([oracle.kron_apply(X[t], R1, R2) for t in range(T)])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


# ------------------------------------------------ the whole transform (Sec. 3.1, Eq. 1) ----

def _tiny_layer():
    cfg = synth.CONFIGS["tiny"]
    return cfg, synth.layer(cfg)


def test_seeded_qr_factors_are_orthogonal():
    for cfg in synth.CONFIGS.values():
        R1, R2 = synth.kron_factors(cfg)
        for R in (R1, R2):
            assert np.max(np.abs(R.T @ R - np.eye(R.shape[0]))) <= 1e-6


def test_rotation_preserves_norms_and_inner_products(oracle):
    cfg, L = _tiny_layer()
    Xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1_f64, L.R2_f64)
    Xf = L.X.astype(np.float64)
    np.testing.assert_allclose(np.linalg.norm(Xr, axis=1), np.linalg.norm(Xf, axis=1), rtol=1e-12)
    np.testing.assert_allclose(Xr @ Xr.T, Xf @ Xf.T, rtol=1e-9, atol=1e-9 * np.max(np.abs(Xf @ Xf.T)))


def test_rotated_product_equals_plain_product(oracle):
    # Eq. 1: X W = (X R)(R^T W), with Flat(W~_R) = W^T R (Sec. 4.2) for the weight side
    cfg, L = _tiny_layer()
    Wt = synth.weights_t(cfg)
    Xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1_f64, L.R2_f64)
    Wr = oracle.rotate(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1_f64, L.R2_f64)
    want = L.X.astype(np.float64) @ Wt.astype(np.float64).T
    got = Xr @ Wr.T
    assert np.max(np.abs(got - want)) <= 1e-9 * np.max(np.abs(want))


def test_rotate_matches_explicit_dense_R_on_small_case(oracle):
    # R = G_1 ... G_P (R1 (x) R2) assembled as one dense matrix by numpy
    g = np.random.default_rng(3)
    n1, n2, T = 4, 6, 5
    K = n1 * n2
    X = g.standard_normal((T, K)).astype(np.float16)
    R1 = synth.random_orthogonal(n1, g)
    R2 = synth.random_orthogonal(n2, g)
    gi = np.array([1, 7, 1, 20], np.int32)     # shares channels: order matters
    gj = np.array([7, 3, 23, 1], np.int32)
    gt = np.array([0.4, -1.3, 2.2, 0.9], np.float64)
    R = np.eye(K)
    for i, j, th in zip(gi, gj, gt):
        R = R @ _explicit_givens(K, int(i), int(j), float(th))
    R = R @ np.kron(R1, R2)
    want = X.astype(np.float64) @ R
    got = oracle.rotate(X, gi, gj, gt, R1, R2)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # a reversed list must give something else (the order is part of the definition)
    other = oracle.rotate(X, gi[::-1], gj[::-1], gt[::-1], R1, R2)
    assert np.max(np.abs(other - want)) > 1e-3


def test_generated_art_angles_are_locally_optimal(oracle):
    """Each Givens angle of the synthetic layers is the minimiser of the pair's infinity norm
    (Lemma 1), checked by brute force over theta on the replayed calibration row."""
    grid = np.linspace(0.0, 2 * math.pi, 100001)
    cg, sg = np.cos(grid), np.sin(grid)
    for name in ("tiny", "attn_proj"):
        cfg = synth.CONFIGS[name]
        X = synth.activations(cfg, min(cfg.T, synth.BLOCK))
        gi, gj, gt = synth.art_pairs(cfg, X)
        assert len(gi) == cfg.P and np.all(gi != gj)
        c = X[int(np.argmax(np.max(np.abs(X.astype(np.float64)), axis=1)))].astype(np.float64)
        for i, j, th in zip(gi, gj, gt):
            a, b = c[i], c[j]
            r = math.hypot(a, b)
            assert abs(a) == np.max(np.abs(c))              # i is the outlier channel
            brute = np.maximum(np.abs(a * cg + b * sg), np.abs(b * cg - a * sg)).min()
            c = oracle.givens_apply(c, int(i), int(j), float(th))
            got = max(abs(c[i]), abs(c[j]))
            assert got <= brute * (1 + 1e-9) and abs(got - r / math.sqrt(2)) <= 1e-6 * r
            assert abs(c[i] - c[j]) <= 2e-6 * r             # the pair is equalised


# ------------------------------------------------------------- Sec. 3.2: quantizer ---------

def _codes(Q):
    """Independent nibble decode (numpy bit operations): low nibble = even channel."""
    lo = (Q & 0xF).astype(np.int16)
    hi = (Q >> 4).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty((Q.shape[0], Q.shape[1] * 2), np.int16)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_quantizer_ties_round_half_up(oracle, dtype):
    # max|z| = 7 => step 1, so z/step + 1/2 is exact: floor(z + 1/2)
    z = np.array([[7.0, 0.5, -0.5, 2.5, -2.5, 6.5, -6.5, -7.0, 1.49, -1.51, 0.0, 3.0]], dtype=dtype)
    Q, s = oracle.quantize_rows(z)
    assert s[0] == 1.0
    assert _codes(Q)[0].tolist() == [7, 1, 0, 3, -2, 7, -6, -7, 1, -2, 0, 3]
    # byte layout: low nibble = even channel, two's complement
    assert Q[0, 0] == (7 | (1 << 4)) and Q[0, 2] == ((-2 & 0xF) | (7 << 4))


def test_quantizer_zero_row_and_scale(oracle):
    z = np.zeros((2, 8))
    z[1] = [0.0, -21.0, 3.0, 1.0, 0.0, 0.0, 10.4, 10.6]
    Q, s = oracle.quantize_rows(z)
    assert s[0] == 1.0 and np.all(Q[0] == 0)
    assert s[1] == np.float32(3.0)
    assert _codes(Q)[1].tolist() == [0, -7, 1, 0, 0, 0, 3, 4]


def test_quantizer_error_bound_and_range(oracle):
    cfg, L = _tiny_layer()
    Xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    for arr in (Xr, Xr.astype(np.float32)):
        Q, s = oracle.quantize_rows(arr)
        q = _codes(Q)
        assert q.min() >= -8 and q.max() <= 7
        err = np.abs(arr.astype(np.float64) - q * s[:, None].astype(np.float64))
        assert np.all(err <= 0.5 * s[:, None] * (1 + 1e-6))
        assert np.all(np.max(np.abs(q), axis=1) == 7)
        np.testing.assert_allclose(s, np.max(np.abs(arr), axis=1) / 7.0, rtol=1e-6)
    assert np.array_equal(oracle.unpack_codes(Q).astype(np.int16), q)


def test_rotation_shrinks_the_quantization_range():
    """Not a parity pin, a sanity check of the recipe: on the outlier-laden synthetic rows the
    transform lowers max|x| / rms(x), which is what makes 4 bits usable (Sec. 3.1)."""
    import oracle
    cfg, L = _tiny_layer()
    Xf = L.X.astype(np.float64)
    Xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    crest = lambda a: np.max(np.abs(a), axis=1) / np.sqrt(np.mean(a * a, axis=1))
    assert np.all(crest(Xr) < 0.5 * crest(Xf))


# --------------------------------------------------------- Eq. 1 on the integer codes ------

def test_gemm_brute_force_and_dequant_closed_form(oracle):
    g = np.random.default_rng(17)
    T, K, N = 5, 64, 7
    Qx = g.integers(0, 256, (T, K // 2), dtype=np.uint8)      # all 16 codes occur, -8 included
    Qw = g.integers(0, 256, (N, K // 2), dtype=np.uint8)
    sx = g.uniform(0.01, 3.0, T).astype(np.float32)
    sw = g.uniform(1e-4, 0.01, N).astype(np.float32)
    Y, acc = oracle.gemm(Qx, sx, Qw, sw)
    want_acc = _codes(Qx).astype(np.int64) @ _codes(Qw).astype(np.int64).T
    assert np.array_equal(acc, want_acc)
    want_Y = (want_acc.astype(np.float64) * sx[:, None].astype(np.float64) * sw[None, :].astype(np.float64))
    assert np.array_equal(Y.view(np.uint16), want_Y.astype(np.float16).view(np.uint16))
    assert oracle.gemm_acc_at(Qx, Qw, 3, 2) == want_acc[3, 2]
    # extreme codes: every product is (-8)(-8) = 64
    Qm = np.full((2, K // 2), 0x88, np.uint8)
    _, accm = oracle.gemm(Qm, np.ones(2, np.float32), Qm, np.ones(2, np.float32))
    assert np.all(accm == 64 * K)


def test_gemm_checksum_invariants(oracle):
    g = np.random.default_rng(23)
    T, K, N = 9, 96, 11
    Qx = g.integers(0, 256, (T, K // 2), dtype=np.uint8)
    Qw = g.integers(0, 256, (N, K // 2), dtype=np.uint8)
    _, acc = oracle.gemm(Qx, np.ones(T, np.float32), Qw, np.ones(N, np.float32))
    cx, cw = _codes(Qx).astype(np.int64), _codes(Qw).astype(np.int64)
    assert np.array_equal(acc.sum(axis=0), cx.sum(axis=0) @ cw.T)
    assert np.array_equal(acc.sum(axis=1), cx @ cw.sum(axis=0))


def test_quantized_layer_approximates_fp_product(oracle):
    """End to end on the tiny layer: rotate + int4 + GEMM + dequant lands near X W (Eq. 1 holds
    up to the two 4-bit roundings), and a wrong rotation on one side does not."""
    cfg, L = _tiny_layer()
    Wt = synth.weights_t(cfg)
    ref = L.X.astype(np.float64) @ Wt.astype(np.float64).T

    def run(gi, gj, gt, R1, R2):
        Qx, sx = oracle.quantize_rows(oracle.rotate(L.X, gi, gj, gt, R1, R2))
        Qw, sw = oracle.prepare_weights(Wt, gi, gj, gt, R1, R2)
        Y, _ = oracle.gemm(Qx, sx, Qw, sw)
        return np.linalg.norm(Y.astype(np.float64) - ref) / np.linalg.norm(ref)

    e_rot = run(L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    assert e_rot < 0.3
    # activations rotated, weights not: the product is no longer X W
    Qx, sx = oracle.quantize_rows(oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2))
    none = np.zeros(0)
    Qw, sw = oracle.prepare_weights(Wt, none, none, none, np.eye(cfg.n1), np.eye(cfg.n2))
    Y, _ = oracle.gemm(Qx, sx, Qw, sw)
    assert np.linalg.norm(Y.astype(np.float64) - ref) / np.linalg.norm(ref) > 0.9


# ------------------------------------------------------------------ Alg. 1 -----------------

def test_kron_factor_values(oracle):
    # worked by hand from Alg. 1: n2 = power of two dividing n closest to sqrt(n), strict "<"
    assert oracle.kron_factor(4096) == (64, 64)
    assert oracle.kron_factor(11008) == (86, 128)
    assert oracle.kron_factor(512) == (32, 16)
    assert oracle.kron_factor(8192) == (128, 64)
    assert oracle.kron_factor(5120) == (80, 64)
    assert oracle.kron_factor(77) == (77, 1)
    assert oracle.kron_factor(1) == (1, 1)


# ------------------------------------------------- weight-only variant (W4A16, Table B.3) --

def test_rotate_f16_is_the_rotation_rounded_once(oracle):
    """The 16-bit activations are the fp64 rotated rows rounded to the nearest fp16: checked
    against numpy's own float64 -> float16 conversion (correctly rounded, ties to even)."""
    L = synth.layer(synth.CONFIGS["tiny"], 5)
    xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    xh = oracle.rotate_f16(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    assert xh.dtype == np.float16 and np.array_equal(xh, xr.astype(np.float16))
    # an exact tie between two fp16 neighbours goes to the even one
    lib = oracle._load()
    out = np.empty((1, 2), np.uint16)
    ties = np.array([[1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11]])
    lib.sqo_round_rows_to_half(ties.ctypes.data, 1, 2, out.ctypes.data, 2)
    assert list(out.view(np.float16)[0]) == [1.0, 1.0 + 2.0 ** -9]


def test_gemm_w4a16_against_brute_force(oracle):
    """Y = fp16(sw * sum_k x q) against a plain numpy evaluation on decoded codes (code -8
    included), non-square so that a transposed operand cannot hide; Eq. 1 with exact activations
    reproduces X W' for the dequantized weights W'."""
    g = np.random.default_rng(8)
    T, K, N = 5, 64, 7
    X = (g.standard_normal((T, K)) * 3).astype(np.float16)
    Qw = synth.random_codes(N, K, 9)
    sw = g.uniform(1e-3, 1e-2, N).astype(np.float32)
    Y, m = oracle.gemm_w4a16(X, Qw, sw, want_abs_sum=True)
    lo = (Qw & 0xF).astype(np.int64)
    hi = (Qw >> 4).astype(np.int64)
    q = np.empty((N, K), np.int64)
    q[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    q[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    assert q.min() == -8 and q.max() == 7
    Wd = q.astype(np.float64) * sw.astype(np.float64)[:, None]           # dequantized W^T
    want = X.astype(np.float64) @ Wd.T
    got = Y.astype(np.float64)
    assert np.all(np.abs(got - want) <= 2.0 ** -11 * np.abs(want) + 1e-300)     # one rounding to fp16
    assert np.allclose(m, np.abs(X.astype(np.float64)) @ np.abs(Wd).T, rtol=1e-12)
    # one hand-worked element: x = (1.5, -2), codes (-8, 7), step 0.5 -> 0.5 (1.5 * -8 + -2 * 7) = -13
    y1 = oracle.gemm_w4a16(np.array([[1.5, -2.0]], np.float16), np.array([[0x78]], np.uint8), np.array([0.5], np.float32))
    assert y1[0, 0] == np.float16(-13.0)


def test_weight_only_pipeline_reproduces_xw(oracle):
    """Eq. 1 with only the weights quantized: (X R)(R^T W) with 4-bit R^T W stays close to X W,
    and the only error is the weight quantizer's (the rotation is orthogonal): with the step
    halved (codes from a finer grid emulated by scaling W) the error halves."""
    cfg = synth.CONFIGS["tiny"]
    L = synth.layer(cfg)
    Wt = synth.weights_t(cfg, 64)
    ref = L.X.astype(np.float64) @ Wt.astype(np.float64).T
    xh = oracle.rotate_f16(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Qw, sw = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Y = oracle.gemm_w4a16(xh, Qw, sw).astype(np.float64)
    err = np.linalg.norm(Y - ref) / np.linalg.norm(ref)
    assert err < 0.2
    # the same weights through the unquantized rotated product: (X R)(R^T W) = X W up to the fp16
    # roundings of R1, R2 and of X R (R is orthogonal only to 1e-3 after its fp16 rounding)
    wr = oracle.rotate(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    exact = xh.astype(np.float64) @ wr.T
    assert np.linalg.norm(exact - ref) / np.linalg.norm(ref) < 5e-3
    # and the quantized product differs from that one by the weight rounding only: |dW| <= s/2
    bound = np.abs(xh.astype(np.float64)) @ np.tile((sw.astype(np.float64) / 2)[None, :], (cfg.K, 1))
    assert np.all(np.abs(Y - exact) <= bound * (1 + 1e-6) + 2.0 ** -10 * np.abs(exact))


# ------------------------------- quantizer with b bits and a clipping ratio; 3-bit storage --

def test_variant_quantizer_reduces_to_the_four_bit_one(oracle):
    """b = 4, ratio 1 is the quantizer of Sec. 3.2 as sqo_quantize_rows writes it: same bytes,
    same steps, on rotated outlier-laden rows."""
    cfg, L = _tiny_layer()
    Xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Q0, s0 = oracle.quantize_rows(Xr)
    Q1, s1 = oracle.quantize_rows_variant(Xr, 4, 1.0)
    assert np.array_equal(Q0, Q1) and np.array_equal(s0, s1)


def test_variant_quantizer_hand_worked_rows(oracle):
    # three bits: levels -4 .. 3, step max|z| / 3 = 1; ties go up (floor(z + 1/2))
    z = np.array([[3.0, -3.0, 1.4, 1.6, -0.5, 0.5, 2.5, -2.5]])
    Q, s = oracle.quantize_rows_variant(z, 3, 1.0)
    assert s[0] == 1.0 and _codes(Q)[0].tolist() == [3, -3, 1, 2, 0, 1, 3, -2]
    # ratio 1/2 at four bits: step 0.5 * 14 / 7 = 1; what lies beyond the levels is clamped to -8, 7
    z = np.array([[14.0, -14.0, 9.0, -12.0, 3.5, -3.5, 0.49, 7.5, -8.5, -8.6]])
    Q, s = oracle.quantize_rows_variant(z, 4, 0.5)
    assert s[0] == 1.0 and _codes(Q)[0].tolist() == [7, -8, 7, -8, 4, -3, 0, 7, -8, -8]
    # two bits: levels -2 .. 1, step max|z|
    Q, s = oracle.quantize_rows_variant(np.array([[2.0, -2.0, 0.9, -1.1, -3.1, 1.1]]), 2, 1.0)
    assert s[0] == np.float32(3.1) and _codes(Q)[0].tolist() == [1, -1, 0, 0, -1, 0]
    # zero row
    Q, s = oracle.quantize_rows_variant(np.zeros((1, 4)), 3, 0.7)
    assert s[0] == 1.0 and np.all(Q == 0)
    for bad in [(1, 1.0), (5, 1.0), (4, 0.0), (4, 1.5), (4, float("nan"))]:
        with pytest.raises(ValueError):
            oracle.quantize_rows_variant(np.ones((1, 4)), *bad)


@pytest.mark.parametrize("bits,ratio", [(3, 1.0), (4, 0.8), (3, 0.6), (2, 1.0)])
def test_variant_quantizer_error_bound_and_range(oracle, bits, ratio):
    """Inside the clipping range the rounding error is at most half a step (Sec. 3.2: the
    boundaries sit at (k + 1/2) D); outside, the code is the nearest end level; the step is
    ratio max|z| / (2^(b-1) - 1)."""
    cfg, L = _tiny_layer()
    Xr = oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)
    Q, s = oracle.quantize_rows_variant(Xr, bits, ratio)
    q = _codes(Q).astype(np.float64)
    top, bottom = 2 ** (bits - 1) - 1, -(2 ** (bits - 1))
    assert q.min() >= bottom and q.max() <= top
    s64 = s.astype(np.float64)[:, None]
    np.testing.assert_allclose(s, ratio * np.max(np.abs(Xr), axis=1) / top, rtol=1e-6)
    inside = (Xr >= (bottom - 0.5) * s64) & (Xr < (top + 0.5) * s64)
    assert np.all(np.abs(Xr - q * s64)[inside] <= 0.5 * s64.repeat(Xr.shape[1], 1)[inside] * (1 + 1e-6))
    assert np.all(q[Xr >= (top + 0.5) * s64] == top) and np.all(q[Xr < (bottom - 0.5) * s64] == bottom)
    if ratio == 1.0:
        assert inside.all() and np.all(np.max(np.abs(q), axis=1) >= top)
    else:
        assert not inside.all()              # the case does clip


def test_w3_storage_matches_the_hand_worked_bytes(oracle):
    import os
    codes = np.full(64, -4, np.int64)
    want = np.zeros(24, np.uint8)
    with open(os.path.join(os.path.dirname(__file__), "golden", "w3_storage_example.txt")) as f:
        for line in f:
            parts = line.split()
            if not parts or parts[0].startswith("#"):
                continue
            if parts[0] == "code":
                codes[int(parts[1])] = int(parts[2])
            else:
                want[int(parts[1])] = int(parts[2], 16)
    nib = (codes & 0xF).astype(np.uint8)
    Q = (nib[0::2] | (nib[1::2] << 4))[None, :]
    Q3 = oracle.pack_w3(Q)
    assert Q3.shape == (1, 24) and Q3[0].tolist() == want.tolist()
    assert np.array_equal(oracle.unpack_w3(Q3), Q)


def test_w3_storage_is_a_bijection_on_every_position(oracle):
    """Every (position, value) changes its own bits only: a row with one code raised from -4 to
    v has exactly popcount(v + 4) bits set, bit sets of different positions are disjoint, and
    packing then unpacking returns every row; three bits per code exactly (3K/8 bytes)."""
    K = 128
    seen = np.zeros((K, 3 * K // 8), np.uint8)
    for k in range(K):
        codes = np.full(K, -4, np.int64)
        codes[k] = 3
        nib = (codes & 0xF).astype(np.uint8)
        Q = (nib[0::2] | (nib[1::2] << 4))[None, :]
        seen[k] = oracle.pack_w3(Q)[0]
        assert int(np.unpackbits(seen[k]).sum()) == 3
        for v in range(-4, 4):
            codes[k] = v
            nib = (codes & 0xF).astype(np.uint8)
            Qv = (nib[0::2] | (nib[1::2] << 4))[None, :]
            pv = oracle.pack_w3(Qv)[0]
            assert int(np.unpackbits(pv).sum()) == bin(v + 4).count("1")
            assert np.all((pv & ~seen[k]) == 0)
    assert np.all(np.bitwise_or.reduce(seen, axis=0) == 0xFF)          # every stored bit is used ...
    assert int(np.unpackbits(seen).sum()) == 3 * K                          # ... by exactly one position
    # codes 64 .. 127 live in the second 24 bytes, laid out like the first
    assert np.all(seen[:64, 24:] == 0) and np.array_equal(seen[64:, 24:], seen[:64, :24])
    g = np.random.default_rng(3)
    codes = g.integers(-4, 4, size=(5, 256))
    nib = (codes & 0xF).astype(np.uint8)
    Q = nib[:, 0::2] | (nib[:, 1::2] << 4)
    assert np.array_equal(oracle.unpack_w3(oracle.pack_w3(Q)), Q)
    bad = Q.copy()
    bad[0, 0] = 0x07                                                     # code 7 is not a 3-bit code
    with pytest.raises(ValueError):
        oracle.pack_w3(bad)


def test_gemm_w3a16_is_the_weight_only_product_on_three_bit_codes(oracle):
    g = np.random.default_rng(12)
    T, K, N = 3, 64, 5
    X = g.standard_normal((T, K)).astype(np.float16)
    codes = g.integers(-4, 4, size=(N, K))
    nib = (codes & 0xF).astype(np.uint8)
    Q = nib[:, 0::2] | (nib[:, 1::2] << 4)
    sw = g.uniform(1e-2, 1e-1, N).astype(np.float32)
    Y = oracle.gemm_w3a16(X, oracle.pack_w3(Q), sw).astype(np.float64)
    want = X.astype(np.float64) @ (codes * sw.astype(np.float64)[:, None]).T
    assert np.all(np.abs(Y - want) <= 2.0 ** -11 * np.abs(want) + 1e-300)


def test_decode_layout_matches_hand_worked_positions_and_is_a_bijection(oracle):
    import os
    K, N = 512, 33
    Kb = K // 2
    g = np.random.default_rng(17)
    Q = g.integers(0, 256, size=(N, Kb), dtype=np.uint8)
    Qt = oracle.tile_weights_decode(Q)
    assert Qt.shape == (2 * 32 * Kb,)
    with open(os.path.join(os.path.dirname(__file__), "golden", "decode_layout_positions.txt")) as f:
        rows = [tuple(int(v) for v in line.split()) for line in f if line.strip() and not line.startswith("#")]
    assert len(rows) == 9
    for n, j, at in rows:
        one = np.zeros((N, Kb), np.uint8)
        one[n, j] = 0xC3
        t = oracle.tile_weights_decode(one)
        assert t[at] == 0xC3 and np.count_nonzero(t) == 1, (n, j, at)
    # a permutation of the N * Kb bytes into distinct places; the padding channels stay zero
    idx = oracle.tile_weights_decode(np.ones((N, Kb), np.uint8))
    assert int(idx.sum()) == N * Kb and set(np.unique(idx)) == {0, 1}
    assert np.array_equal(oracle.untile_weights_decode(Qt, N, K), Q)
    # every 16-byte unit is 16 consecutive bytes of one channel's row
    tags = (np.arange(N * Kb, dtype=np.int64) // 16).reshape(N, Kb)
    low, high = oracle.tile_weights_decode((tags & 0xFF).astype(np.uint8)), oracle.tile_weights_decode((tags >> 8).astype(np.uint8))
    units = (low.astype(np.int64) | (high.astype(np.int64) << 8)).reshape(-1, 16)
    assert np.all(units == units[:, :1])
    with pytest.raises(ValueError):
        oracle.tile_weights_decode(np.zeros((4, 64), np.uint8))       # K = 128 is not a multiple of 256
