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
