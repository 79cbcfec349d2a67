"""Helpers shared by the GPU parity tests: device marshalling and the parity metrics.

Tolerances (from the benchmark spec, restated where they are used):
  * rotated activations: per token  max_k|g - o| / max_k|o| <= 1e-5  and  ||G - O||_F / ||O||_F <= 1e-5
  * per-token steps:     |s_gpu - s_or| / s_or <= 1e-5
  * codes:               every |q_gpu - q_or| <= 1, and at most 1e-4 of all codes differ
  * int32 accumulators:  bit-exact given identical codes
  * fp16 Y:              per row ||dy||_2 / ||y||_2 <= 1e-2; given identical codes, within 1 fp16 ulp
"""
from __future__ import annotations

import numpy as np

XROT_TOL = 1e-5
SCALE_TOL = 1e-5
CODE_FLIP_FRACTION = 1e-4
Y_ROW_TOL = 1e-2


def codes_of(Q: np.ndarray) -> np.ndarray:
    """Nibble decode with numpy bit operations (low nibble = even channel), int16 [rows, K]."""
    lo = (Q & 0xF).astype(np.int16)
    hi = (Q >> 4).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty((Q.shape[0], Q.shape[1] * 2), np.int16)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


def dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def host(t) -> np.ndarray:
    return t.detach().cpu().numpy()


def run_rotate_quantize(L, X=None, want_xrot=True, xrot_rows=None):
    """Call the library on layer L (optionally on other rows X).  -> (Q, scales, xrot) numpy;
    xrot_rows: bring back only these rows of the rotated activations (full-size runs)."""
    import torch
    import paper_2511_22316_amd as sq
    X = L.X if X is None else X
    T, K = X.shape
    dX, dR1, dR2 = dev(X), dev(L.R1), dev(L.R2)
    Q = torch.empty((T, K // 2), dtype=torch.uint8, device="cuda")
    s = torch.empty((T,), dtype=torch.float32, device="cuda")
    xr = torch.empty((T, K), dtype=torch.float32, device="cuda") if want_xrot else None
    sq.sq_rotate_quantize(dX, L.giv_i, L.giv_j, L.giv_theta, dR1, dR2, Q, s, xr)
    torch.cuda.synchronize()
    # The same call through the prepared form of R1, R2 must give the same bits: every check the
    # caller makes on the result then holds for both entry points.
    n1, n2 = L.R1.shape[0], L.R2.shape[0]
    prepared = torch.full((sq.sq_prepared_rotation_bytes(n1, n2) + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    sq.sq_prepare_rotation(dR1, dR2, prepared)
    Qp = torch.full_like(Q, 0x5A)
    sp = torch.full_like(s, -1.0)
    xp = torch.full_like(xr, -7.0) if want_xrot else None
    sq.sq_rotate_quantize_prepared(dX, L.giv_i, L.giv_j, L.giv_theta, prepared, n1, n2, Qp, sp, xp)
    torch.cuda.synchronize()
    assert torch.all(prepared[-64:] == 0xA5), "sq_prepare_rotation wrote past its stated size"
    assert torch.equal(Qp, Q) and torch.equal(sp, s), "prepared rotation: codes or steps differ from the plain call"
    if want_xrot:
        assert torch.equal(xp, xr), "prepared rotation: rotated activations differ from the plain call"
    if want_xrot and xrot_rows is not None:
        xr = xr[torch.from_numpy(np.asarray(xrot_rows, dtype=np.int64)).cuda()]
    return host(Q), host(s), (host(xr) if want_xrot else None)


def run_gemm(Qx, sx, Qw, sw, want_acc=True):
    import torch
    import paper_2511_22316_amd as sq
    T, N = Qx.shape[0], Qw.shape[0]
    Y = torch.empty((T, N), dtype=torch.float16, device="cuda")
    acc = torch.empty((T, N), dtype=torch.int32, device="cuda") if want_acc else None
    sq.sq_w4a4_gemm(dev(Qx), dev(sx), dev(Qw), dev(sw), Y, acc)
    torch.cuda.synchronize()
    return host(Y), (host(acc) if want_acc else None)


def check_rotation(xrot_gpu: np.ndarray, xrot_or: np.ndarray) -> None:
    d = xrot_gpu.astype(np.float64) - xrot_or
    per_tok = np.max(np.abs(d), axis=1) / np.maximum(np.max(np.abs(xrot_or), axis=1), 1e-300)
    assert per_tok.max() <= XROT_TOL, f"rotated activations: worst per-token max error {per_tok.max():.3e}"
    fro = np.linalg.norm(d) / max(np.linalg.norm(xrot_or), 1e-300)
    assert fro <= XROT_TOL, f"rotated activations: Frobenius error {fro:.3e}"


def check_codes(Q_gpu, s_gpu, Q_or, s_or) -> float:
    rel = np.abs(s_gpu.astype(np.float64) - s_or) / s_or
    assert rel.max() <= SCALE_TOL, f"per-token steps: worst relative error {rel.max():.3e}"
    qg, qo = codes_of(Q_gpu), codes_of(Q_or)
    assert qg.min() >= -8 and qg.max() <= 7
    diff = np.abs(qg - qo)
    assert diff.max() <= 1, "a code differs by more than one step"
    frac = float(np.count_nonzero(diff)) / diff.size
    assert frac <= CODE_FLIP_FRACTION, f"{frac:.3e} of the codes differ"
    return frac


def half_ulp_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in units of fp16 spacing between two float16 arrays (finite values)."""
    def key(x):
        u = x.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a) - key(b))
