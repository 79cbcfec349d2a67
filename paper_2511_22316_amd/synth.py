"""Seeded synthetic LLaMA-shaped layers: the inputs of the W4A4 hot path.

This module only *draws inputs*.  It holds none of the hot path's arithmetic
(no Kronecker product, no quantizer, no GEMM) and imports neither the HIP
binding nor the CPU oracle, so both sides can be fed the same bytes.

The shapes follow LLaMA hidden / intermediate sizes; the outlier structure
follows the paper's description of activations (Sec. 3.1): a few "massive
outlier" channels of huge magnitude on every token, plus moderate "normal
outliers" spread over many entries.  They stand in for the calibration and
evaluation activations of the paper's models, which are not available here.

Everything is generated in blocks of ``BLOCK`` rows, each block from its own
``numpy`` PCG64 stream keyed by (seed, tensor id, block index), so any subset
of rows can be re-drawn without materialising the full tensor.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

BLOCK = 256
_FP16_MAX = 65504.0
_TAG_X, _TAG_W, _TAG_R1, _TAG_R2, _TAG_PERM = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int                 # tokens
    n1: int                # Kronecker factor sizes, K = n1 * n2
    n2: int
    N: int                 # output channels
    P: int                 # number of Givens (ART) pairs
    x_dist: str            # "normal" | "student_t3"
    massive: object        # explicit channel tuple, or an int count (seeded permutation)
    massive_scale: float
    normal_frac: float     # Bernoulli probability of a x20 "normal outlier"
    normal_scale: float
    w_std: float
    seed: int

    @property
    def K(self) -> int:
        return self.n1 * self.n2


_BASE_SEED = 20251122

CONFIGS = {
    "tiny": LayerConfig("tiny", 16, 16, 32, 512, 8, "normal", (3, 101), 500.0, 0.01, 20.0, 0.02, _BASE_SEED + 1),
    "attn_proj": LayerConfig("attn_proj", 2048, 64, 64, 4096, 32, "normal", 4, 1000.0, 0.01, 20.0, 0.02, _BASE_SEED + 2),
    "mlp_down": LayerConfig("mlp_down", 2048, 86, 128, 4096, 16, "student_t3", 2, 2000.0, 0.0, 20.0, 0.02, _BASE_SEED + 3),
    "decode": LayerConfig("decode", 8, 64, 128, 28672, 32, "normal", 4, 1000.0, 0.0, 20.0, 0.015, _BASE_SEED + 4),
    "large_prefill": LayerConfig("large_prefill", 8192, 64, 128, 28672, 64, "normal", 8, 1000.0, 0.005, 20.0, 0.015, _BASE_SEED + 5),
}


def _rng(seed: int, tag: int, block: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, tag, block]))


def massive_channels(cfg: LayerConfig) -> np.ndarray:
    """Channel indices that carry the massive outliers."""
    if isinstance(cfg.massive, int):
        return np.sort(_rng(cfg.seed, _TAG_PERM).permutation(cfg.K)[: cfg.massive]).astype(np.int64)
    return np.asarray(cfg.massive, dtype=np.int64)


def _x_block(cfg: LayerConfig, block: int, mch: np.ndarray) -> np.ndarray:
    g = _rng(cfg.seed, _TAG_X, block)
    if cfg.x_dist == "normal":
        x = g.standard_normal((BLOCK, cfg.K))
    elif cfg.x_dist == "student_t3":
        x = g.standard_t(3.0, (BLOCK, cfg.K))
    else:
        raise ValueError(cfg.x_dist)
    if cfg.normal_frac > 0.0:
        hit = g.random((BLOCK, cfg.K)) < cfg.normal_frac
        hit[:, mch] = False
        x = np.where(hit, x * cfg.normal_scale, x)
    x[:, mch] *= cfg.massive_scale
    np.clip(x, -_FP16_MAX, _FP16_MAX, out=x)     # never hand Inf to the path
    return x.astype(np.float16)


def activation_rows(cfg: LayerConfig, rows: Sequence[int]) -> np.ndarray:
    """fp16 [len(rows), K]: the given token rows of X."""
    rows = np.asarray(rows, dtype=np.int64)
    mch = massive_channels(cfg)
    out = np.empty((rows.size, cfg.K), np.float16)
    for b in np.unique(rows // BLOCK):
        blk = _x_block(cfg, int(b), mch)
        sel = np.nonzero(rows // BLOCK == b)[0]
        out[sel] = blk[rows[sel] % BLOCK]
    return out


def activations(cfg: LayerConfig, T: Optional[int] = None) -> np.ndarray:
    """fp16 [T, K] activations X (row = token)."""
    T = cfg.T if T is None else T
    mch = massive_channels(cfg)
    out = np.empty((T, cfg.K), np.float16)
    for b in range((T + BLOCK - 1) // BLOCK):
        lo, hi = b * BLOCK, min(T, (b + 1) * BLOCK)
        out[lo:hi] = _x_block(cfg, b, mch)[: hi - lo]
    return out


def _w_block(cfg: LayerConfig, block: int) -> np.ndarray:
    g = _rng(cfg.seed, _TAG_W, block)
    return (g.standard_normal((BLOCK, cfg.K), dtype=np.float32) * np.float32(cfg.w_std)).astype(np.float16)


def weight_rows_t(cfg: LayerConfig, rows: Sequence[int]) -> np.ndarray:
    """fp16 [len(rows), K]: rows of W^T, i.e. one K-vector per output channel."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((rows.size, cfg.K), np.float16)
    for b in np.unique(rows // BLOCK):
        blk = _w_block(cfg, int(b))
        sel = np.nonzero(rows // BLOCK == b)[0]
        out[sel] = blk[rows[sel] % BLOCK]
    return out


def weights_t(cfg: LayerConfig, N: Optional[int] = None) -> np.ndarray:
    """fp16 [N, K] = W^T (the layout the paper reshapes into W~, Sec. 4.2); entries N(0, w_std)."""
    N = cfg.N if N is None else N
    out = np.empty((N, cfg.K), np.float16)
    for b in range((N + BLOCK - 1) // BLOCK):
        lo, hi = b * BLOCK, min(N, (b + 1) * BLOCK)
        out[lo:hi] = _w_block(cfg, b)[: hi - lo]
    return out


def random_orthogonal(n: int, g: np.random.Generator) -> np.ndarray:
    """Seeded QR of a Gaussian matrix with the sign fix Q diag(sign(diag R)); fp64."""
    q, r = np.linalg.qr(g.standard_normal((n, n)))
    d = np.sign(np.diag(r))
    d[d == 0] = 1.0
    return q * d[None, :]


def kron_factors(cfg: LayerConfig) -> Tuple[np.ndarray, np.ndarray]:
    """(R1 [n1,n1], R2 [n2,n2]) in fp64, orthogonal to ~1e-15.  Round to fp16 before use on
    either side: both the library and the oracle take the fp16 values."""
    return (random_orthogonal(cfg.n1, _rng(cfg.seed, _TAG_R1)),
            random_orthogonal(cfg.n2, _rng(cfg.seed, _TAG_R2)))


def art_pairs(cfg: LayerConfig, X: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Givens list for the layer, drawn the way the paper's ART picks it (Sec. 4.2): on a
    calibration row (the token of X with the largest |entry|), repeat P times: i = channel of
    the largest magnitude, j = channel of the smallest magnitude, angle from Lemma 1, rotate the
    calibration row, go on.  Pairs may share channels, so the list order matters.
    Returns (i int32 [P], j int32 [P], theta float32 [P]); also the (a, b) each angle was made
    for is recoverable by replaying the list."""
    Xf = np.asarray(X, dtype=np.float64)
    c = Xf[int(np.argmax(np.max(np.abs(Xf), axis=1)))].copy()
    gi = np.empty(cfg.P, np.int32)
    gj = np.empty(cfg.P, np.int32)
    gt = np.empty(cfg.P, np.float32)
    for p in range(cfg.P):
        mag = np.abs(c)
        i = int(np.argmax(mag))
        mag[i] = np.inf
        j = int(np.argmin(mag))
        a, b = c[i], c[j]
        theta = np.float32(np.arctan2(b, a) - np.pi / 4.0)
        co, si = np.cos(np.float64(theta)), np.sin(np.float64(theta))
        c[i], c[j] = a * co + b * si, b * co - a * si
        gi[p], gj[p], gt[p] = i, j, theta
    return gi, gj, gt


def random_codes(rows: int, K: int, seed: int) -> np.ndarray:
    """uint8 [rows, K/2]: uniformly random nibble pairs (codes over the full [-8, 7] range)."""
    return _rng(seed, 99).integers(0, 256, size=(rows, K // 2), dtype=np.uint8)


@dataclass
class Layer:
    cfg: LayerConfig
    X: np.ndarray          # fp16 [T, K]
    giv_i: np.ndarray      # int32 [P]
    giv_j: np.ndarray      # int32 [P]
    giv_theta: np.ndarray  # float32 [P]
    R1: np.ndarray         # fp16 [n1, n1]
    R2: np.ndarray         # fp16 [n2, n2]
    R1_f64: np.ndarray     # before fp16 rounding
    R2_f64: np.ndarray


def layer(cfg: LayerConfig, T: Optional[int] = None) -> Layer:
    """Activations, Givens list and Kronecker factors of one layer (weights are drawn
    separately with weights_t / weight_rows_t because they can be large)."""
    X = activations(cfg, T)
    # the calibration row is searched in the first block only, so that a shortened T >= BLOCK
    # and the full T give the same Givens list
    gi, gj, gt = art_pairs(cfg, X[:BLOCK])
    R1, R2 = kron_factors(cfg)
    return Layer(cfg, X, gi, gj, gt, R1.astype(np.float16), R2.astype(np.float16), R1, R2)
