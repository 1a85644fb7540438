"""MI355X-native EDGC hot path: thin Python binding over ``libedgc.so``.

The library (hand-written HIP for gfx950 behind the C ABI of ``include/edgc.h``)
does all the work; this package only marshals arguments.  PyTorch is used by
callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    BF16, F32, Context, EdgcError, EntropyResult, PreparedBatch, RankBounds, RankCost, RankDecision, RankParams,
    RankState, Tensor, entropy_due, fit_eta, lib_path, load_library, rank_bounds, select_rank, stage_ranks, tensor_bypassed,
)
