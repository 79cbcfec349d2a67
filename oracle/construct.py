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

Precision.  Where floating point decides an index (the ART channels, the rank order of the
URT), the decision is taken in fp32, one rounding per operation, in index order -- the
precision of the kernel.  Everything downstream of the decisions is fp64.
"""
from __future__ import annotations

import math

import numpy as np

F32 = np.float32
_INV_SQRT2_F32 = F32(0.70710678118654752440)


def calibration_row(X_f16: np.ndarray) -> int:
    """Row of X with the largest |entry|; ties go to the lowest row."""
    m = np.max(np.abs(np.asarray(X_f16, dtype=np.float32)), axis=1)      # exact in fp32
    return int(np.argmax(m))


def art_select(c, P: int):
    """P ART steps on the calibration vector c.
    -> (i int32 [P], j int32 [P], theta float64 [P], c after the steps (float32))."""
    c = np.array(c, dtype=np.float32)
    gi = np.empty(P, np.int32)
    gj = np.empty(P, np.int32)
    gt = np.empty(P, np.float64)
    for p in range(P):
        mag = np.abs(c)
        i = int(np.argmax(mag))                  # first of the largest
        rest = mag.copy()
        rest[i] = np.inf
        j = int(np.argmin(rest))                 # first of the smallest among the others
        a, b = c[i], c[j]
        # Lemma 1: theta* = atan2(b, a) - pi/4 and (a, b) G(theta*) = (r, r) / sqrt(2)
        gt[p] = math.atan2(float(b), float(a)) - math.pi / 4.0
        r = np.sqrt(a * a + b * b)               # float32 scalars: one rounding per operation
        c[i] = c[j] = r * _INV_SQRT2_F32
        gi[p], gj[p] = i, j
    return gi, gj, gt, c


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


def urt_vectors(c_f32, n1: int, n2: int):
    """(V1, V2 H) in fp32 as the rank decisions see them: means over the other dimension of the
    n1 x n2 view of c, added up in index order; V2 H with the signs of H, added up in index order
    and scaled by 1/sqrt(n2) at the end."""
    Cm = np.asarray(c_f32, dtype=np.float32).reshape(n1, n2)
    V1 = np.cumsum(Cm, axis=1, dtype=np.float32)[:, -1] / F32(n2)
    V2 = np.cumsum(Cm, axis=0, dtype=np.float32)[-1, :] / F32(n1)
    sign = np.sign(hadamard(n2)).astype(np.float32)                       # [a, b] = +-1
    V2H = np.cumsum(V2[:, None] * sign, axis=0, dtype=np.float32)[-1, :] * F32(1.0 / math.sqrt(n2))
    return V1, V2, V2H


def build_rotation(X_f16, n1: int, n2: int, P: int):
    """The whole constructor.  -> dict with the calibration row, the Givens list, the vectors of
    the two URTs, and R1, R2 in fp64 (round to fp16 to compare with the library)."""
    X_f16 = np.asarray(X_f16)
    t = calibration_row(X_f16)
    gi, gj, gt, c = art_select(X_f16[t].astype(np.float32), P)
    V1, V2, V2H = urt_vectors(c, n1, n2)
    R1 = urt(V1)
    R2 = hadamard(n2) @ urt(V2H)
    return dict(row=t, giv_i=gi, giv_j=gj, giv_theta=gt, c=c, V1=V1, V2=V2, V2H=V2H, R1=R1, R2=R2)
