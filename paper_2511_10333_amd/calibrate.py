"""Rank-bound calibration on the GPU at hand (Sec. IV-D-1 of the paper).

Times this library's compress and decompress at a list of candidate ranks on the matrices
of one transformer block (synthetic gradients of the given hidden size), then, for each
network bandwidth given, solves  T_compress + D_compressed/B + T_decompress <= D_original/B
for r_max, derives r_min, and fits T_com(r) = eta r over [r_min, r_max].

    python -m paper_2511_10333_amd.calibrate --hidden 2048 --dtype f32 --gbps 32 100 400

Prints one JSON object.  Needs a GPU and the built library.
"""
from __future__ import annotations

import argparse
import json

import torch

from . import Context, fit_eta, rank_bounds, RankCost


def block_shapes(hidden: int):
    return [(hidden, 3 * hidden), (hidden, hidden), (hidden, 4 * hidden), (4 * hidden, hidden)]


def measure_block(hidden: int, dtype: torch.dtype, ranks, reps: int, seed: int = 0, deferred: bool = True):
    """Sum of the per-matrix costs over the four matrices of a block, per rank."""
    r_cap = max(ranks)
    total = [RankCost(r, 0.0, 0.0, 0.0) for r in ranks]
    gen = torch.Generator(device="cuda").manual_seed(seed)
    for m, n in block_shapes(hidden):
        ctx = Context(0, max_rank=r_cap, max_rows=m, max_cols=n)
        g = (1e-3 * torch.randn((m, n), device="cuda", generator=gen)).to(dtype)
        res = torch.empty((m, n), device="cuda")
        out = torch.empty((m, n), device="cuda", dtype=dtype)
        Q = torch.empty((n, r_cap), device="cuda")
        P = torch.empty((m, r_cap), device="cuda")
        for acc, c in zip(total, ctx.measure_rank_costs(g, res, Q, P, out, ranks, reps, deferred=deferred)):
            acc.t_compress += c.t_compress
            acc.t_decompress += c.t_decompress
            acc.bytes_compressed += c.bytes_compressed
        del ctx, g, res, out, Q, P
    return total


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--hidden", type=int, default=2048)
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--ranks", type=int, nargs="+", default=[4, 8, 16, 32, 64, 128])
    ap.add_argument("--gbps", type=float, nargs="+", default=[32.0, 100.0, 400.0, 8568.0],
                    help="network bandwidths in Gbit/s (8568 = seven xGMI links of 153 GB/s)")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--explicit-residual", action="store_true",
                    help="time the form that stores E between steps instead of the deferred one")
    ap.add_argument("--divisor", type=float, default=4.0, help="r_min = ceil(r_max / divisor), 4..6")
    a = ap.parse_args(argv)
    dtype = torch.float32 if a.dtype == "f32" else torch.bfloat16
    costs = measure_block(a.hidden, dtype, sorted(a.ranks), a.reps, deferred=not a.explicit_residual)
    elem = 4 if a.dtype == "f32" else 2
    d_orig = float(sum(m * n for m, n in block_shapes(a.hidden)) * elem)
    report = {"hidden": a.hidden, "dtype": a.dtype, "residual": "explicit" if a.explicit_residual else "deferred", "bytes_original": d_orig, "reps": a.reps,
              "costs": [{"rank": c.rank, "t_compress_us": 1e6 * c.t_compress,
                         "t_decompress_us": 1e6 * c.t_decompress,
                         "bytes_compressed": c.bytes_compressed} for c in costs],
              "bandwidths": []}
    for gbps in a.gbps:
        bw = gbps * 1e9 / 8.0
        b = rank_bounds(costs, d_orig, bw, a.divisor)
        entry = {"gbps": gbps, "t_uncompressed_us": 1e6 * b.t_uncompressed, "r_max": b.r_max,
                 "r_min": b.r_min, "t_com_us": [1e6 * t for t in b.t_com], "eta_us": None,
                 "mape_percent": None}
        inside = [(c.rank, t) for c, t in zip(costs, b.t_com) if b.r_min <= c.rank <= b.r_max]
        if inside:
            eta, mape = fit_eta([r for r, _ in inside], [t for _, t in inside])
            entry["eta_us"], entry["mape_percent"] = 1e6 * eta, mape
        report["bandwidths"].append(entry)
    print(json.dumps(report))
    return report


if __name__ == "__main__":
    main()
