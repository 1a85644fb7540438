"""Helpers for the GPU parity tests: host <-> device copies, bf16 views, error norms."""
import numpy as np
import torch

import paper_2511_10333_amd as edgc

_ctx = {}


def ctx(max_bins=1 << 20, max_rank=128, max_rows=20480, max_cols=20480):
    key = (max_bins, max_rank, max_rows, max_cols)
    if key not in _ctx or not getattr(_ctx[key], "_h", None):     # (re)create when a test closed it
        _ctx[key] = edgc.Context(0, max_bins, max_rank, max_rows, max_cols)
    return _ctx[key]


def to_dev(a: np.ndarray) -> torch.Tensor:
    """float32 -> float32 tensor; uint16 (bf16 bits) -> bfloat16 tensor (same bits)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def rel_fro(a, b) -> float:
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def elementwise_ratio(got, want, P, Q, chunk=1024) -> float:
    """max over (i, j) of |got_ij - want_ij| / (||P_i|| ||Q_j||): the reconstruction error of every single
    element against the scale Cauchy-Schwarz gives it (P: m x r, Q: n x r of the reference)."""
    npn = np.linalg.norm(np.asarray(P, dtype=np.float64), axis=1)
    nq = np.linalg.norm(np.asarray(Q, dtype=np.float64), axis=1)
    worst = 0.0
    for i0 in range(0, got.shape[0], chunk):
        d = np.abs(np.asarray(got[i0:i0 + chunk], dtype=np.float64) - np.asarray(want[i0:i0 + chunk], dtype=np.float64))
        den = npn[i0:i0 + chunk, None] * nq[None, :]
        ok = den > 0
        if ok.any():
            worst = max(worst, float((d[ok] / den[ok]).max()))
        if (~ok).any():
            assert float(d[~ok].max()) == 0.0, "non-zero reconstruction where a factor row is zero"
    return worst


# Element-wise bar on the reconstruction, in units of ||p_i|| ||q_j||: the Frobenius tolerance for fp32; with bf16
# gradients the two sides may round an operand of a term, or the output, to neighbouring bf16 values (their
# fp32 factors agree to ~1e-5, not to the bit): one bf16 ulp (2^-8 relative) on either operand and on the
# output, 3 * 2^-8 = 1.17e-2 of ||p_i|| ||q_j|| at most by Cauchy-Schwarz.
ELEMENTWISE_TOL = {"f32": 1e-3, "bf16": 3.0 / 256.0}
