"""CPU-side checks of the product library: it loads, exports every symbol the
public header declares, and its host-only rank selector agrees with the oracle."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "edgc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(edgc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = edgc.load_library()
    names = _declared_functions()
    assert {"edgc_create", "edgc_destroy", "edgc_last_error", "edgc_entropy_estimate",
            "edgc_sample_indices", "edgc_select_rank", "edgc_init_q", "edgc_compress",
            "edgc_decompress"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/edgc.h but not exported"


def test_struct_sizes_match_the_header_layout():
    from paper_2511_10333_amd import binding as b
    assert ctypes.sizeof(b._EntropyResult) == 48
    assert ctypes.sizeof(b._RankDecision) == 32
    assert ctypes.sizeof(b._RankState) == 32
    assert ctypes.sizeof(b._RankCost) == 32
    assert ctypes.sizeof(b._RankBounds) == 16
    assert ctypes.sizeof(b._DevicePeaks) == 40            # copy, read, mfma, bytes, write


def _both(prm_kwargs, windows):
    st_o, st_p = orc.RankState(), edgc.RankState()
    out = []
    for H, iters in windows:
        d_o = orc.select_rank(st_o, H, iters, orc.RankParams(**prm_kwargs))
        d_p = edgc.select_rank(st_p, H, iters, edgc.RankParams(**prm_kwargs))
        out.append((d_o, d_p))
        assert (st_o.have_ref, st_o.compressing, st_o.r_prev, st_o.iters_seen) == \
               (st_p.have_ref, st_p.compressing, st_p.r_prev, st_p.iters_seen)
        assert st_o.H_ref == pytest.approx(st_p.H_ref, abs=1e-12)
    return out


@pytest.mark.parametrize("shape", [(512, 512), (256, 1024), (1920, 640), (4096, 4096)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_rank_matches_oracle_on_random_entropy_walks(shape, seed):
    rng = np.random.default_rng(seed)
    m, n = shape
    prm = dict(m=m, n=n, r_min=4, r_max=64, step_limit=8, allowed=[4, 8, 16, 32, 64], eta=0.25,
               total_iters=400, min_warmup_frac=0.10, r_ref=int(rng.choice([0, 4, 32])))
    H = -8.0
    windows = []
    for _ in range(20):
        H += float(rng.normal(-0.01, 0.05))
        windows.append(([H + float(e) for e in rng.normal(0, 0.01, 5)], 20))
    for d_o, d_p in _both(prm, windows):
        assert d_o.rank == d_p.rank
        assert d_o.r_unclamped == d_p.r_unclamped
        assert d_o.H_mean == pytest.approx(d_p.H_mean, abs=1e-12)
        assert d_o.T_com == d_p.T_com


@pytest.mark.parametrize("bounds", [(6, 48), (5, 31), (9, 100), (16, 16)])
def test_select_rank_snaps_inside_the_bounds_like_the_oracle(bounds):
    # allowed ranks outside [r_min, r_max] are never emitted (r_max of Sec. IV-D-1 is a hard bound)
    rng = np.random.default_rng(7)
    r_min, r_max = bounds
    prm = dict(m=512, n=768, r_min=r_min, r_max=r_max, step_limit=8, allowed=[4, 8, 16, 32, 64, 128], eta=0.5,
               total_iters=0, min_warmup_frac=0.0, r_ref=0)
    H, windows = -6.0, []
    for k in range(40):
        H += float(rng.normal(-0.08 if k < 20 else 0.12, 0.1))
        windows.append(([H], 10))
    seen = set()
    for d_o, d_p in _both(prm, windows):
        assert d_o.rank == d_p.rank and d_o.r_unclamped == d_p.r_unclamped and d_o.T_com == d_p.T_com
        if d_p.rank:
            assert r_min <= d_p.rank <= r_max
            seen.add(d_p.rank)
    assert seen


def test_select_rank_hand_table_and_warmup():
    prm = dict(m=512, n=512, r_min=16, r_max=64, step_limit=8, eta=0.5, total_iters=100,
               min_warmup_frac=0.10)
    st = edgc.RankState()
    p = edgc.RankParams(**prm)
    assert edgc.select_rank(st, [0.0], 5, p).rank == 0          # reference window
    assert edgc.select_rank(st, [-3.0], 4, p).rank == 0         # 9 < 10 iterations
    ranks = [edgc.select_rank(st, [-3.0], 5, p).rank for _ in range(8)]
    assert ranks == [56, 48, 40, 32, 24, 16, 16, 16]
    assert [edgc.select_rank(st, [1.0], 5, p).rank for _ in range(7)] == [24, 32, 40, 48, 56, 64, 64]


def test_select_rank_rejects_bad_input():
    st = edgc.RankState()
    for kw in [dict(r_max=0), dict(r_max=1000), dict(r_min=65), dict(allowed=[8, 4]), dict(r_min=0),
               dict(r_min=33, r_max=63, allowed=[4, 8, 16, 32, 64])]:
        a = dict(m=512, n=512, r_min=4, r_max=64); a.update(kw)
        with pytest.raises(edgc.EdgcError) as e:
            edgc.select_rank(st, [0.0], 1, edgc.RankParams(**a))
        assert e.value.code == -1
    with pytest.raises(edgc.EdgcError) as e:
        edgc.select_rank(st, [math.nan], 1, edgc.RankParams(512, 512, 4, 64))
    assert e.value.code == -5
    with pytest.raises(edgc.EdgcError):
        edgc.select_rank(st, [], 1, edgc.RankParams(512, 512, 4, 64))
