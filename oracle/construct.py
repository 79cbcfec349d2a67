"""CPU oracle of the closed-form rotation constructor (Sec. 4.2: ART, URT, Alg. 1, composition).

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing in the product imports it.
Plain numpy, one step of the paper per function, no blocking or fusion.

What is computed (the readings of the paper that are not forced by its text are marked READING;
they are the same ones the library documents for ``sq_build_rotation``):

  calibration vector  READING: the token row of X with the largest |entry| (ties: lowest row).
  ART (Sec. 4.2 "Alignment Rotation Transformation", multi-step as in the "ART steps" study)
        P times: i = channel of largest magnitude, j = channel of smallest magnitude (j != i,
        ties: lowest channel), angle from Lemma 1 for (a, b) = (c_i, c_j), after which both
        channels hold r / sqrt(2) (Lemma 1).  READING: the pairs index the K-channel space and
        are returned as a Givens list (they are not folded into a Kronecker factor).
  URT (Sec. 4.2 "Uniformity Rotation Transformation")
        target U: the centred uniform template q_k = (2k - n - 1) / n handed out by the rank
        order of V and scaled to the norm of V;  R_map, R'_map: n - 1 plane rotations each that
        take V and U to ||V|| e_1;  R^U = R_map R'_map^T, so that V R^U = U.
        READING (the paper leaves the chain open): the rotation that zeroes entry k acts in
        the plane (k - 1, k), k = n - 1 down to 1.
  vectors the two URTs are built from   READING ("different dimensions of the activation"):
        with C the n1 x n2 view of the calibration vector after ART, V1 = row means of C,
        V2 = column means of C; the second URT sees V2 H because H acts first.
  composition (Sec. 4.2 "The Overall SingleQuant Method")   R1 = R^U_1,  R2 = H R^U_2.
        READING: the paper prints the left factor transposed, for matrices that act on column
        vectors; Lemma 1 and the URT property are stated for row vectors, and under Eq. 18
        (rows: x -> rvec(R1^T X_mat R2)) the factor that sends the columns of X_mat to their
        uniform target is R^U_1 itself.

Precision.  Everything is fp64, the decisions included: the paper defines the ART channels and
the rank order of the URT over the reals.

Close calls.  Multi-step ART produces them by itself: a massive entry a rotated against a tiny
entry b leaves a (1 + b^2 / 2a^2) / sqrt(2) in both channels, so the halves of two outliers, or
of one outlier met twice, differ only in their 13th to 16th digit, and which of them is "the
largest" next is then not a property of the method but of the last bits.  (With a = 19712 and
b = 1e-4 the difference is below fp64 resolution altogether: two such halves come out "equal" or
not depending on how the square root was evaluated.)  ``art_select`` therefore reports its closest call (``margin``: the smallest relative distance between a winner
and the best candidate that is not tied with it by construction -- equal inputs, or the two
outputs of one step, which the index rule decides in any arithmetic), and it can be told to
``follow`` another implementation's choices: a followed choice is accepted if it is the oracle's
own or if its magnitude lies within the relative ``band`` of the oracle's winner and is not a
tie by construction, and is counted as a departure; any other choice raises.  The rank order
of the URT has a margin of its own (``rank_margin``).
"""
from __future__ import annotations

import math

import numpy as np


def calibration_row(X_f16: np.ndarray) -> int:
    """Row of X with the largest |entry|; ties go to the lowest row."""
    m = np.max(np.abs(np.asarray(X_f16, dtype=np.float32)), axis=1)      # exact in fp32
    return int(np.argmax(m))


def _tied(mag: np.ndarray, origin: np.ndarray, k: int) -> np.ndarray:
    """Channels that hold the magnitude of channel k by construction, in any arithmetic: equal
    values that are both inputs, or both the result of the same ART step.  (Equal values of
    different origin are a coincidence of rounding, not a tie.)"""
    return (mag == mag[k]) & (origin == origin[k])


def _runner_up_gap(mag: np.ndarray, origin: np.ndarray, won: int, largest: bool, skip: int = -1) -> float:
    """Relative distance from mag[won] to the nearest candidate that is not tied with it by
    construction (those the index decides); inf if there is none."""
    keep = ~_tied(mag, origin, won)
    if skip >= 0:
        keep[skip] = False
    if not keep.any():
        return math.inf
    other = float(mag[keep].max() if largest else mag[keep].min())
    top = max(float(mag[won]), other)
    return 0.0 if top == 0.0 else abs(float(mag[won]) - other) / top


def _smallest_other(mag: np.ndarray, i: int) -> int:
    rest = mag.copy()
    rest[i] = np.inf
    return int(np.argmin(rest))                  # first of the smallest among the others


def art_select(c, P: int, follow=None, band: float = 0.0):
    """P ART steps on the calibration vector c.
    follow: None, or (i [P], j [P]) chosen elsewhere, taken instead of the oracle's own channels
    where they are within ``band`` of them (see the module text); ValueError otherwise.
    -> (i int32 [P], j int32 [P], theta float64 [P], c after the steps, margin, departures)."""
    c = np.array(c, dtype=np.float64)
    origin = np.full(c.size, -1)                 # step that wrote the channel, -1: still the input
    gi = np.empty(P, np.int32)
    gj = np.empty(P, np.int32)
    gt = np.empty(P, np.float64)
    margin = math.inf
    departures = 0
    for p in range(P):
        mag = np.abs(c)
        i = own_i = int(np.argmax(mag))          # first of the largest
        j = own_j = _smallest_other(mag, i)
        margin = min(margin, _runner_up_gap(mag, origin, i, True), _runner_up_gap(mag, origin, j, False, skip=i))
        if follow is not None:
            fi, fj = int(follow[0][p]), int(follow[1][p])
            if fi != i:
                # among channels tied by construction the lowest index wins: not a close call
                if not (0 <= fi < c.size and mag[fi] >= mag[i] * (1.0 - band) and not _tied(mag, origin, i)[fi]):
                    raise ValueError(f"ART step {p}: channel {fi} is not the largest (channel {i} is)")
                i = fi
                j = _smallest_other(mag, i)
            if fj != j:
                if not (0 <= fj < c.size and fj != i and mag[fj] <= mag[j] * (1.0 + band)
                        and not _tied(mag, origin, j)[fj]):
                    raise ValueError(f"ART step {p}: channel {fj} is not the smallest (channel {j} is)")
                j = fj
            departures += (i, j) != (own_i, own_j)
        a, b = c[i], c[j]
        # Lemma 1: theta* = atan2(b, a) - pi/4 and (a, b) G(theta*) = (r, r) / sqrt(2)
        gt[p] = math.atan2(b, a) - math.pi / 4.0
        c[i] = c[j] = math.hypot(a, b) / math.sqrt(2.0)
        origin[i] = origin[j] = p
        gi[p], gj[p] = i, j
    return gi, gj, gt, c, margin, departures


def uniform_template(n: int) -> np.ndarray:
    """q_k = (2k - n - 1) / n, k = 1 .. n."""
    k = np.arange(1, n + 1, dtype=np.float64)
    return (2.0 * k - n - 1.0) / n


def uniform_target(V) -> np.ndarray:
    """U: template entries handed out by the rank order of V (ascending, ties by index), scaled
    so that ||U|| = ||V||."""
    V = np.asarray(V, dtype=np.float64)
    n = V.size
    q = uniform_template(n)
    order = np.argsort(V, kind="stable")         # pi: V[order[0]] <= V[order[1]] <= ...
    U = np.empty(n)
    U[order] = np.linalg.norm(V) / np.linalg.norm(q) * q
    return U


def map_to_e1(V) -> np.ndarray:
    """R_map: a product of n - 1 plane rotations with V R_map = ||V|| e_1.  Entry k is zeroed by a
    rotation in the plane (k - 1, k), from the last entry upwards."""
    v = np.array(V, dtype=np.float64)
    n = v.size
    R = np.eye(n)
    for k in range(n - 1, 0, -1):
        h = math.hypot(v[k - 1], v[k])
        if h == 0.0:
            continue
        co, si = v[k - 1] / h, v[k] / h
        G = np.array([[co, -si], [si, co]])      # (x, y) G = (x co + y si, -x si + y co)
        R[:, [k - 1, k]] = R[:, [k - 1, k]] @ G
        v[[k - 1, k]] = v[[k - 1, k]] @ G
    return R


def urt(V) -> np.ndarray:
    """R^U = R_map R'_map^T with V R^U = U."""
    return map_to_e1(V) @ map_to_e1(uniform_target(V)).T


def hadamard(n: int) -> np.ndarray:
    """Normalised Hadamard matrix of Sylvester's doubling construction (n a power of two)."""
    if n < 1 or n & (n - 1):
        raise ValueError("n must be a power of two")
    H = np.ones((1, 1))
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]]) / math.sqrt(2.0)
    return H


def rank_margin(V) -> float:
    """Smallest gap between two different entries of V, relative to the largest |entry|
    (inf if all entries are equal)."""
    v = np.sort(np.asarray(V, dtype=np.float64))
    gaps = np.diff(v)
    gaps = gaps[gaps > 0]
    return math.inf if gaps.size == 0 else float(gaps.min() / np.max(np.abs(v)))


def urt_vectors(c, n1: int, n2: int):
    """(V1, V2, V2 H): means over the other dimension of the n1 x n2 view of c; the vector of the
    second URT goes through H first, because H acts first in R2 = H R^U_2."""
    Cm = np.asarray(c, dtype=np.float64).reshape(n1, n2)
    V1 = Cm.mean(axis=1)
    V2 = Cm.mean(axis=0)
    return V1, V2, V2 @ hadamard(n2)


def build_rotation(X_f16, n1: int, n2: int, P: int, follow=None, band: float = 0.0):
    """The whole constructor.  -> dict with the calibration row, the Givens list, the vectors of
    the two URTs, R1, R2 in fp64 (round to fp16 to compare with the library), ``art_margin`` and
    ``rank_margin`` (the closest calls among its ART and rank-order decisions) and
    ``departures`` (see ``art_select`` for ``follow`` and ``band``)."""
    X_f16 = np.asarray(X_f16)
    t = calibration_row(X_f16)
    gi, gj, gt, c, art_margin, departures = art_select(X_f16[t].astype(np.float64), P, follow, band)
    V1, V2, V2H = urt_vectors(c, n1, n2)
    R1 = urt(V1)
    R2 = hadamard(n2) @ urt(V2H)
    return dict(row=t, giv_i=gi, giv_j=gj, giv_theta=gt, c=c, V1=V1, V2=V2, V2H=V2H, R1=R1, R2=R2,
                art_margin=art_margin, rank_margin=min(rank_margin(V1), rank_margin(V2H)), departures=departures)
