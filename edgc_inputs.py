"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: only random tensors with the shapes,
value distributions and structure of the workloads (low-rank-plus-noise layer
gradients, a Laplace mixture with outliers for flat buffers).  They stand in
for the real GPT-2 / BERT training gradients the paper measured on, which are
not available here.  bf16 tensors are ``uint16`` arrays of raw bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even (input preparation)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def orthonormal_factors(m: int, n: int, k: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Random orthonormal U (m x k), V (n x k): thin QR of seeded Gaussians."""
    rng = np.random.default_rng([seed, 0x0F])
    U, _ = np.linalg.qr(rng.standard_normal((m, k)))
    V, _ = np.linalg.qr(rng.standard_normal((n, k)))
    return U.astype(np.float64), V.astype(np.float64)


def lowrank_plus_noise(m: int, n: int, k: int, decay: float, noise_sigma: float, seed: int,
                       dtype: str = "f32", noise_seed: int | None = None,
                       factors: Tuple[np.ndarray, np.ndarray] | None = None) -> np.ndarray:
    """M = U diag(decay^i, i<k) V^T + noise_sigma * Z, as float32 or bf16 bits."""
    U, V = factors if factors is not None else orthonormal_factors(m, n, k, seed)
    s = decay ** np.arange(k, dtype=np.float64)
    M = (U * s) @ V.T
    rng = np.random.default_rng([seed if noise_seed is None else noise_seed, 0x5A])
    M += noise_sigma * rng.standard_normal((m, n))
    M32 = M.astype(np.float32)
    return to_bf16_bits(M32) if dtype == "bf16" else M32


def exact_rank(m: int, n: int, r: int, seed: int) -> np.ndarray:
    """A float32 matrix of exact rank r (up to fp32 rounding of its entries)."""
    rng = np.random.default_rng([seed, 0xE0])
    A = rng.standard_normal((m, r))
    B = rng.standard_normal((r, n))
    return (A @ B / np.sqrt(r)).astype(np.float32)


def gaussian(n: int, sigma: float, seed: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 0x6A])
    return (sigma * rng.standard_normal(n)).astype(np.float32)


def laplace_mixture(n: int, seed: int, dtype: str = "f32", scale: float = 1e-3,
                    outlier_frac: float = 1e-3, outlier_scale: float = 1e-1,
                    block: int = 1 << 24) -> np.ndarray:
    """Flat gradient buffer: Laplace(0, scale) with a fraction of outliers at 100x scale.

    Generated block by block (each block seeded by its index) so any prefix of a
    larger buffer is reproducible without generating the rest.
    """
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    for b0 in range(0, n, block):
        b1 = min(n, b0 + block)
        rng = np.random.default_rng([seed, 0x1A, b0 // block])
        x = rng.laplace(0.0, scale, b1 - b0)
        mask = rng.random(b1 - b0) < outlier_frac
        x[mask] *= outlier_scale / scale
        x32 = x.astype(np.float32)
        out[b0:b1] = to_bf16_bits(x32) if dtype == "bf16" else x32
    return out


@dataclass(frozen=True)
class LayerSpec:
    name: str
    m: int
    n: int


def gpt_block(hidden: int) -> List[LayerSpec]:
    """The four 2-D gradients of one GPT-style block, row-major (in x out)."""
    return [LayerSpec("qkv", hidden, 3 * hidden), LayerSpec("attn_proj", hidden, hidden),
            LayerSpec("mlp_up", hidden, 4 * hidden), LayerSpec("mlp_down", 4 * hidden, hidden)]


# The workloads named by the benchmark contract, in its order.
WORKLOADS: Dict[str, dict] = {
    "cfg1_1024sq_r4": dict(layers=[LayerSpec("square", 1024, 1024)], dtype="f32", k=64, decay=0.90,
                           noise=1e-4, stride=100, chunk=64, bins=256, rank=4, seed=0),
    "cfg2_gpt_h2048_r16": dict(layers=gpt_block(2048), dtype="f32", k=256, decay=0.95, noise=1e-4,
                               stride=100, chunk=64, bins=1024, rank=16, seed=0),
    "cfg4_gpt_h5120_bf16": dict(layers=gpt_block(5120), dtype="bf16", k=512, decay=0.97, noise=1e-4,
                                stride=100, chunk=64, bins=1024, rank=64, seed=0),
    "cfg5_stage_h4096": dict(layers=gpt_block(4096), dtype="f32", k=1024, decay=0.90, noise=1e-4,
                             stride=100, chunk=64, bins=1024, rank=64, seed=0),
    # the whole pipeline stage of that configuration: 8 layers, 32 tensors, 1.61e9 elements; the
    # 8 layers carry the same four seeded gradients (generating 32 distinct ones takes minutes)
    "cfg5_stage8_h4096": dict(layers=gpt_block(4096), repeat=8, dtype="f32", k=1024, decay=0.90, noise=1e-4,
                              stride=100, chunk=64, bins=1024, rank=64, seed=0),
}


def workload_matrices(name: str, scale_hidden: int | None = None) -> List[Tuple[LayerSpec, np.ndarray]]:
    """Materialise every layer gradient of a named workload (optionally at a smaller hidden)."""
    w = WORKLOADS[name]
    out = []
    for li, spec in enumerate(w["layers"]):
        m, n = spec.m, spec.n
        if scale_hidden is not None:
            base = min(s.m for s in w["layers"])
            m, n = m * scale_hidden // base, n * scale_hidden // base
        k = min(w["k"], m, n)
        g = lowrank_plus_noise(m, n, k, w["decay"], w["noise"], w["seed"] + 17 * li, w["dtype"])
        out.append((LayerSpec(spec.name, m, n), g))
    rep = w.get("repeat", 1)
    if rep > 1:
        out = [(LayerSpec("L%d.%s" % (layer, spec.name), spec.m, spec.n), g)
               for layer in range(rep) for spec, g in out]
    return out
