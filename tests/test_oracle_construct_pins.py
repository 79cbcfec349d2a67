"""Pins of the rotation-constructor oracle (ART, URT, Hadamard, composition of Sec. 4.2) against
what the paper and the mathematics fix: the closed forms of Lemma 1, the URT property
V R^U = U, hand-worked cases, scipy's Hadamard matrix, brute force, and the Kronecker identity of
Eq. 18 closed over a rank-one calibration matrix.  None compares the oracle with itself.  CPU only.
"""
import math

import numpy as np
import pytest
import scipy.linalg

from oracle import construct as oc


# ------------------------------------------------------------------ ART -------------------

def test_art_hand_worked_steps(oracle):
    # |c| = (3, 0.5, 4, 1): step 1 takes i = 2 (largest), j = 1 (smallest): r = sqrt(16.25);
    # then the largest is r/sqrt(2) = 2.85.. < 3, so step 2 takes i = 0 and j = 3 (|c_3| = 1 is
    # now the smallest), r = sqrt(10)
    c0 = np.array([3.0, -0.5, -4.0, 1.0])
    gi, gj, gt, c, margin, _ = oc.art_select(c0, 2)
    assert list(gi) == [2, 0] and list(gj) == [1, 3]
    assert gt[0] == pytest.approx(math.atan2(-0.5, -4.0) - math.pi / 4, abs=1e-15)
    assert gt[1] == pytest.approx(math.atan2(1.0, 3.0) - math.pi / 4, abs=1e-15)
    e1, e2 = math.sqrt(16.25 / 2), math.sqrt(10.0 / 2)
    assert np.allclose(c, [e2, e1, e1, e2], rtol=1e-15)
    # closest calls, by hand: step 1, largest 4 against 3 (gap 1/4), smallest 0.5 against 1 (1/2);
    # step 2, largest 3 against sqrt(8.125) = 2.850.. (the two equal entries), smallest 1 against
    # 2.850..: the tightest is (3 - 2.850..) / 3
    assert margin == pytest.approx((3.0 - e1) / 3.0, rel=1e-12)


def test_art_ties_go_to_the_lowest_channel(oracle):
    gi, gj, _, _, margin, _ = oc.art_select(np.array([1.0, -7.0, 7.0, 0.25, -0.25, 2.0]), 1)
    assert (gi[0], gj[0]) == (1, 3)
    # exact ties are decided by the index and do not count as close calls: 7 against 2, 0.25 against 1
    assert margin == pytest.approx(min(5.0 / 7.0, 0.75), rel=1e-12)
    # largest and smallest may not be the same channel even if every entry is equal
    gi, gj, _, _, margin, _ = oc.art_select(np.full(5, 2.0), 1)
    assert (gi[0], gj[0]) == (0, 1) and margin == math.inf


def test_margins_flag_decisions_that_hang_on_the_last_digits(oracle):
    gi, _, _, _, margin, _ = oc.art_select(np.array([5.0, 5.0 * (1 + 1e-13), 0.1, 1.0]), 1)
    assert gi[0] == 1 and margin == pytest.approx(1e-13, rel=1e-2)
    assert oc.rank_margin([1.0, 3.0, 3.0 + 3e-12, -2.0]) == pytest.approx(1e-12, rel=1e-3)
    assert oc.rank_margin([2.0, 2.0, 2.0]) == math.inf


def test_following_other_choices_is_allowed_only_inside_the_band(oracle):
    """Two outliers whose halves differ in the 13th digit: either may be called the largest, and
    a follower inside the band is taken and counted; anything else is refused -- a channel
    outside the band, an exactly equal magnitude at a higher index (the index rule is not a
    close call), the largest channel as its own partner."""
    c0 = np.array([5.0, 0.01, 5.0 * (1 + 1e-13), 0.02, 1.0, 0.01])
    gi, gj, _, c_own, margin, dep = oc.art_select(c0, 1)
    assert (gi[0], gj[0], dep) == (2, 1, 0) and margin == pytest.approx(1e-13, rel=1e-2)
    gi, gj, gt, c, _, dep = oc.art_select(c0, 1, follow=([0], [1]), band=1e-12)
    assert (gi[0], gj[0], dep) == (0, 1, 1)
    assert gt[0] == pytest.approx(math.atan2(0.01, 5.0) - math.pi / 4, abs=1e-15)
    assert c[0] == c[1] == pytest.approx(math.sqrt((25.0 + 1e-4) / 2), rel=1e-15) and c[2] == c0[2]
    _, _, _, c, _, dep = oc.art_select(c0, 1, follow=([2], [1]), band=1e-12)
    assert dep == 0 and np.array_equal(c, c_own)
    for bad in (([0], [1], 1e-14), ([4], [1], 1e-12), ([2], [5], 1e-12), ([2], [3], 1e-12), ([2], [2], 1e-12)):
        with pytest.raises(ValueError):
            oc.art_select(c0, 1, follow=(bad[0], bad[1]), band=bad[2])
    # the two outputs of one step are tied by construction: after step 1 channels 2 and 1 hold the
    # same value, step 2 must take the lower one, whatever the band
    with pytest.raises(ValueError):
        oc.art_select(c0, 2, follow=([2, 2], [1, 5]), band=1e-3)
    gi, gj, _, _, _, dep = oc.art_select(c0, 2, follow=([2, 0], [1, 5]), band=1e-12)
    assert list(gi) == [2, 0] and dep == 0          # 5 > 5 (1 + 1e-13) / sqrt 2: channel 0 is next, no close call
    # equal values of different origin are a coincidence of rounding: either index may follow
    c1 = np.array([8.0, 0.0, math.hypot(8.0, 0.0) / math.sqrt(2.0), 0.5, 0.25])
    _, _, _, c, margin, _ = oc.art_select(c1, 1)    # channels 0, 1 <- 8 / sqrt 2, beside an input of that value
    assert c[0] == c[1] == c[2] and margin > 0.25
    gi, _, _, _, margin, dep = oc.art_select(c1, 2, follow=([0, 2], [1, 4]), band=1e-12)
    assert list(gi) == [0, 2] and dep == 1 and margin == 0.0


def test_art_list_replayed_as_givens_rotations_gives_the_same_vector(oracle):
    """The closed-form update (both channels <- r/sqrt 2) must be what the Givens rotation of the
    returned (i, j, theta) does: replay the list with the oracle's Givens routine, whose sign
    convention is pinned against an explicit matrix elsewhere."""
    g = np.random.default_rng(3)
    c0 = g.standard_normal(300) * np.where(g.random(300) < 0.02, 200.0, 1.0)
    P = 24
    gi, gj, gt, c, _, _ = oc.art_select(c0, P)
    v = c0.copy()
    peak = [np.max(np.abs(v))]
    for p in range(P):
        v = oracle.givens_apply(v, int(gi[p]), int(gj[p]), float(gt[p]))
        assert abs(v[gi[p]] - v[gj[p]]) <= 1e-13 * abs(v[gi[p]])       # equalised
        peak.append(np.max(np.abs(v)))
    assert np.allclose(v, c, rtol=1e-12, atol=0)
    assert abs(np.linalg.norm(v) - np.linalg.norm(c0)) <= 1e-12 * np.linalg.norm(v)
    assert all(b <= a * (1 + 1e-12) for a, b in zip(peak, peak[1:]))   # the peak never grows
    assert peak[-1] < 0.5 * peak[0]                                   # and the outliers are spread


def test_art_each_angle_is_the_brute_force_minimiser(oracle):
    g = np.random.default_rng(4)
    c0 = g.standard_normal(64) * np.where(g.random(64) < 0.05, 50.0, 1.0)
    gi, gj, gt, _, _, _ = oc.art_select(c0, 6)
    v = c0.copy()
    grid = np.linspace(0.0, 2 * math.pi, 100001)
    for p in range(6):
        a, b = v[gi[p]], v[gj[p]]
        r = math.hypot(a, b)
        worst = np.maximum(np.abs(a * np.cos(grid) + b * np.sin(grid)), np.abs(b * np.cos(grid) - a * np.sin(grid)))
        assert worst.min() >= r / math.sqrt(2) - 1e-9 * r
        t = gt[p]
        assert max(abs(a * math.cos(t) + b * math.sin(t)), abs(b * math.cos(t) - a * math.sin(t))) <= r / math.sqrt(2) * (1 + 1e-6)
        v = oracle.givens_apply(v, int(gi[p]), int(gj[p]), float(t))


# ------------------------------------------------------------------ URT -------------------

@pytest.mark.parametrize("n", [2, 3, 16, 86, 128])
def test_uniform_template_norm_closed_form(n):
    q = oc.uniform_template(n)
    assert np.dot(q, q) == pytest.approx((n * n - 1) / (3.0 * n), rel=1e-13)
    assert q[0] == pytest.approx((1 - n) / n) and q[-1] == pytest.approx((n - 1) / n)
    assert abs(q.sum()) < 1e-12                                        # centred
    assert np.allclose(np.diff(q), 2.0 / n)                            # evenly spread


def test_uniform_target_hand_worked():
    # V = (0.3, -2, 5): ranks 2, 1, 3 -> template (-2/3, 0, 2/3) lands as (0, -2/3, 2/3), scaled
    V = np.array([0.3, -2.0, 5.0])
    U = oc.uniform_target(V)
    scale = np.linalg.norm(V) / math.sqrt(8.0 / 9.0)
    assert np.allclose(U, scale * np.array([0.0, -2.0 / 3.0, 2.0 / 3.0]), atol=1e-14)
    # n = 2: U = ||V|| (-1, 1)/sqrt 2 in rank order
    assert np.allclose(oc.uniform_target(np.array([4.0, -3.0])), 5.0 * np.array([1.0, -1.0]) / math.sqrt(2))
    # equal entries: the lower index takes the lower rank
    U = oc.uniform_target(np.array([1.0, 1.0, 1.0]))
    assert U[0] < U[1] < U[2]


@pytest.mark.parametrize("n,seed", [(2, 0), (5, 1), (64, 2), (86, 3), (128, 4)])
def test_urt_property_orthogonality_rank_and_norm(n, seed):
    g = np.random.default_rng(seed)
    V = g.standard_normal(n) * np.where(g.random(n) < 0.1, 20.0, 1.0)
    R = oc.urt(V)
    U = V @ R
    assert np.max(np.abs(R.T @ R - np.eye(n))) <= 1e-12
    assert np.linalg.norm(U) == pytest.approx(np.linalg.norm(V), rel=1e-13)
    assert np.array_equal(np.argsort(U, kind="stable"), np.argsort(V, kind="stable"))      # rank order kept
    srt = np.sort(U)
    assert np.allclose(np.diff(srt), srt[1] - srt[0], rtol=1e-9)                            # evenly spread
    assert abs(U.sum()) <= 1e-10 * np.linalg.norm(V)                                        # centred
    assert np.allclose(U, oc.uniform_target(V), atol=1e-11 * np.linalg.norm(V))
    # the flattening the paper is after: the peak-to-rms ratio of a uniform vector is below sqrt 3
    assert np.max(np.abs(U)) / (np.linalg.norm(U) / math.sqrt(n)) <= math.sqrt(3.0) + 1e-9


def test_map_to_e1_is_a_chain_of_plane_rotations():
    g = np.random.default_rng(9)
    V = g.standard_normal(7)
    R = oc.map_to_e1(V)
    e1 = np.zeros(7)
    e1[0] = np.linalg.norm(V)
    assert np.allclose(V @ R, e1, atol=1e-13)
    assert np.max(np.abs(R.T @ R - np.eye(7))) <= 1e-13
    assert np.linalg.det(R) == pytest.approx(1.0, abs=1e-12)           # rotations only, no reflection
    # n - 1 rotations in the planes (k-1, k), last plane first: row r of the product reaches no
    # further than column r + 1 (lower Hessenberg)
    assert np.max(np.abs(np.triu(R, 2))) == 0.0
    # zeros in V are no obstacle, and the zero vector gives the identity
    V0 = np.array([0.0, 0.0, 3.0, 0.0, -4.0])
    assert np.allclose(V0 @ oc.map_to_e1(V0), [5, 0, 0, 0, 0], atol=1e-14)
    assert np.array_equal(oc.map_to_e1(np.zeros(4)), np.eye(4))
    assert np.array_equal(oc.urt(np.zeros(4)), np.eye(4))


# ------------------------------------------------------------------ Hadamard --------------

@pytest.mark.parametrize("n", [1, 2, 4, 32, 64, 128, 256])
def test_hadamard_matches_scipy(n):
    H = oc.hadamard(n)
    assert np.allclose(H, scipy.linalg.hadamard(n) / math.sqrt(n), atol=1e-15)
    assert np.max(np.abs(H @ H.T - np.eye(n))) <= 1e-13
    with pytest.raises(ValueError):
        oc.hadamard(3 * n)


# ------------------------------------------------------------------ the whole constructor --

def test_urt_vectors_are_plain_means(oracle):
    g = np.random.default_rng(11)
    c = g.standard_normal(16 * 32)
    V1, V2, V2H = oc.urt_vectors(c, 16, 32)
    # written out entry by entry, independent of numpy's reductions
    for p in range(16):
        assert V1[p] == pytest.approx(math.fsum(c[p * 32 + q] for q in range(32)) / 32, abs=1e-15)
    for q in range(32):
        assert V2[q] == pytest.approx(math.fsum(c[p * 32 + q] for p in range(16)) / 16, abs=1e-15)
    assert np.allclose(V2H, V2 @ (scipy.linalg.hadamard(32) / math.sqrt(32)), rtol=0, atol=1e-14)


@pytest.mark.parametrize("n1,n2", [(4, 8), (16, 32), (12, 16)])
def test_constructor_flattens_a_rank_one_calibration_matrix(oracle, n1, n2):
    """If the n1 x n2 view of the calibration vector is u v^T, its means are multiples of u and v,
    and by Eq. 18 the rotated vector must be the outer product of the two uniform targets --
    evaluated here through the oracle's own Kronecker routine (pinned against a dense Kronecker
    product elsewhere), so a transposed factor or a Hadamard matrix on the wrong side fails."""
    g = np.random.default_rng(n1 * n2)
    u = g.standard_normal(n1) + 0.3
    v = g.standard_normal(n2) * np.where(g.random(n2) < 0.2, 10.0, 1.0) + 0.2
    row = np.outer(u, v).ravel().astype(np.float16)
    X = np.stack([row * np.float16(0.5), row, row * np.float16(-0.25)])           # row 1 has the peak
    out = oc.build_rotation(X, n1, n2, 0)
    assert out["row"] == 1
    Cm = row.astype(np.float64).reshape(n1, n2)
    got = oracle.kron_apply(row.astype(np.float64), out["R1"], out["R2"]).reshape(n1, n2)
    # exact expectation from the definition alone: V1 = row means, V2 = column means, H acts first
    V1, V2 = Cm.mean(axis=1), Cm.mean(axis=0)
    H = scipy.linalg.hadamard(n2) / math.sqrt(n2)
    # u v^T = V1^T V2 / mean(u v^T), hence R1^T (u v^T) R2 = U1^T U2 / mean(u v^T).  The entries of
    # the calibration row are fp16 roundings of u_p v_q (relative error 2^-11 each), which moves
    # any entry of the rotated matrix by at most 2^-11 ||C||_F.
    U1, U2 = oc.uniform_target(out["V1"]), oc.uniform_target(out["V2H"])
    want = np.outer(U1, U2) / Cm.mean()
    assert np.max(np.abs(got - want)) <= 1.5e-3 * np.linalg.norm(Cm)
    assert np.allclose(out["V1"], V1, rtol=0, atol=1e-13 * np.max(np.abs(V1)))
    assert np.allclose(out["V2H"], V2 @ H, rtol=0, atol=1e-13 * np.max(np.abs(V2)) * math.sqrt(n2))
    for R in (out["R1"], out["R2"]):
        assert np.max(np.abs(R.T @ R - np.eye(R.shape[0]))) <= 1e-12
    # the point of it all: each uniform target has a peak-to-rms ratio below sqrt 3, so the peak of
    # the rotated calibration vector is below 3 times its rms
    assert np.max(np.abs(got)) <= 3.0 * np.linalg.norm(Cm) / math.sqrt(n1 * n2) * (1 + 2e-3)


def test_constructor_on_a_synthetic_layer_reduces_the_peak(oracle):
    from paper_2511_22316_amd import synth
    cfg = synth.CONFIGS["tiny"]
    X = synth.activations(cfg, 16)
    out = oc.build_rotation(X, cfg.n1, cfg.n2, 8)
    assert out["row"] == int(np.argmax(np.max(np.abs(X.astype(np.float64)), axis=1)))
    assert len(set(zip(out["giv_i"], out["giv_j"]))) >= 2 and np.all(out["giv_i"] != out["giv_j"])
    # first pair: the massive channel of the calibration row and its smallest entry
    c0 = X[out["row"]].astype(np.float64)
    assert out["giv_i"][0] == int(np.argmax(np.abs(c0)))
    rest = np.abs(c0)
    rest[out["giv_i"][0]] = np.inf
    assert out["giv_j"][0] == int(np.argmin(rest))
    R1h, R2h = out["R1"].astype(np.float16), out["R2"].astype(np.float16)
    xr = oracle.rotate(X, out["giv_i"], out["giv_j"], out["giv_theta"].astype(np.float32), R1h, R2h)
    before = np.max(np.abs(X.astype(np.float64)), axis=1) / np.sqrt(np.mean(X.astype(np.float64) ** 2, axis=1))
    after = np.max(np.abs(xr), axis=1) / np.sqrt(np.mean(xr ** 2, axis=1))
    assert np.median(after) < 0.5 * np.median(before)                 # peak-to-rms of the tokens drops
    assert np.allclose(np.linalg.norm(xr, axis=1), np.linalg.norm(X.astype(np.float64), axis=1), rtol=2e-3)
