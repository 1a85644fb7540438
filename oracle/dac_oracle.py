"""Oracle for the host arithmetic of the Dynamic Alignment Compressor (test infrastructure).

Plain Python floats (fp64), one statement per step of the paper's text, no code shared with
the library.  Only tests, the smoke check and the bench's CPU-baseline leg may import this.

What each function follows, and the readings taken where the paper leaves a choice:

* ``rank_bounds``  -- Sec. IV-D-1, the inequality  T_compress + D_compressed/B + T_decompress
  <= D_original/B.  Candidates are scanned in ascending rank; the first rank that violates the
  inequality closes the scan, and r_max is the last rank before it (0 when even the smallest
  candidate does not pay).  The footnote puts r_min between r_max/6 and r_max/4: r_min is
  ceil(r_max / divisor) with the divisor a caller's choice in [4, 6], and never below 1.
* ``fit_eta``      -- Sec. IV-D-1, T_com(r) = eta * r.  The paper does not say how eta is
  fitted: least squares through the origin, eta = sum(r T) / sum(r^2); the error it quotes is
  the mean absolute percentage error, 100 * mean(|T - eta r| / T).
* ``stage_ranks``  -- Sec. IV-D-4, Algorithm 2: stage 1 keeps its rank; stage i >= 2 gets the
  rank whose predicted time equals T_com(stage 1) + (i-1) * T_microBack, clamped to the rank
  bounds.  A rank is an integer: the largest integer whose predicted time does not exceed the
  stage's budget (floor, with 1e-9 of slack against T/eta landing just under an integer), and
  with an allowed set the largest allowed rank not above it (the smallest allowed rank when
  none is).
* ``entropy_due``  -- Sec. IV-B, iteration sampling rate alpha: within a window the entropy is
  measured once every 1/alpha iterations; reading: at window-relative iterations 0, 1/alpha,
  2/alpha, ...
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple


def rank_bounds(costs: Sequence[Tuple[int, float, float, float]], bytes_original: float,
                bandwidth: float, r_min_divisor: float):
    """costs: (rank, T_compress [s], T_decompress [s], D_compressed [bytes]) in ascending rank.
    Returns (r_max, r_min, T_uncompressed, [T_com per candidate])."""
    if not costs or bandwidth <= 0 or bytes_original <= 0 or not (4.0 <= r_min_divisor <= 6.0):
        raise ValueError("rank_bounds: bad arguments")
    t_plain = bytes_original / bandwidth
    t_com = []
    for rank, t_c, t_d, d_c in costs:
        t_com.append(t_c + d_c / bandwidth + t_d)
    r_max = 0
    prev = 0
    for (rank, _, _, _), t in zip(costs, t_com):
        if rank <= prev:
            raise ValueError("rank_bounds: ranks must ascend")
        prev = rank
    for (rank, _, _, _), t in zip(costs, t_com):
        if t <= t_plain:
            r_max = rank
        else:
            break
    r_min = 0 if r_max == 0 else max(1, math.ceil(r_max / r_min_divisor))
    return r_max, r_min, t_plain, t_com


def fit_eta(ranks: Sequence[int], t_com: Sequence[float]):
    """Returns (eta, MAPE in percent)."""
    if len(ranks) == 0 or len(ranks) != len(t_com):
        raise ValueError("fit_eta: bad arguments")
    num = 0.0
    den = 0.0
    for r, t in zip(ranks, t_com):
        num += float(r) * t
        den += float(r) * float(r)
    eta = num / den
    ape = 0.0
    for r, t in zip(ranks, t_com):
        ape += abs(t - eta * r) / t
    return eta, 100.0 * ape / len(ranks)


def stage_ranks(r_stage1: int, t_microback: float, eta: float, r_min: int, r_max: int,
                n_stages: int, allowed: Optional[Sequence[int]] = None):
    """Returns ([rank per stage], [predicted T_com per stage])."""
    if eta <= 0 or n_stages < 1 or r_min < 1 or r_min > r_max or t_microback < 0:
        raise ValueError("stage_ranks: bad arguments")
    t1 = eta * r_stage1
    ranks: List[int] = [r_stage1]
    for i in range(2, n_stages + 1):
        budget = t1 + (i - 1) * t_microback
        r = math.floor(budget / eta + 1e-9)
        r = max(r_min, min(r_max, r))
        if allowed:
            below = [a for a in allowed if a <= r]
            r = max(below) if below else min(allowed)
        ranks.append(int(r))
    return ranks, [eta * r for r in ranks]


def entropy_due(iter_in_window: int, period: int) -> bool:
    if period < 1:
        raise ValueError("entropy_due: period must be >= 1")
    return iter_in_window % period == 0
