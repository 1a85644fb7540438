"""ctypes binding with the same names as the C ABI (``include/edgc.h``).

Argument marshalling only: every step of the path runs inside the library's
kernels.  There is no fallback: if ``libedgc.so`` is missing or fails to load,
importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

F32, BF16 = 0, 1
OK, EINVAL, ENOMEM, EHIP, ENOTIMPL, ENONFINITE = 0, -1, -2, -3, -4, -5

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    return os.path.join(_HERE, "libedgc.so")


class EdgcError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str = ""):
        super().__init__(f"{what}: edgc status {code}" + (f" ({detail})" if detail else ""))
        self.code = code


class _EntropyResult(C.Structure):
    _fields_ = [("H_bits", C.c_double), ("h_diff_nats", C.c_double), ("lo", C.c_float),
                ("hi", C.c_float), ("n_sampled", C.c_uint64), ("n_nonfinite", C.c_uint64),
                ("status", C.c_int32), ("_pad", C.c_int32)]


class _RankParams(C.Structure):
    _fields_ = [("m", C.c_uint32), ("n", C.c_uint32), ("r_min", C.c_uint32), ("r_max", C.c_uint32),
                ("step_limit", C.c_uint32), ("allowed", C.POINTER(C.c_uint32)),
                ("n_allowed", C.c_uint32), ("eta", C.c_double), ("total_iters", C.c_uint64),
                ("min_warmup_frac", C.c_double), ("r_ref", C.c_uint32)]


class _RankState(C.Structure):
    _fields_ = [("have_ref", C.c_int32), ("compressing", C.c_int32), ("H_ref", C.c_double),
                ("r_prev", C.c_double), ("iters_seen", C.c_uint64)]


class _RankDecision(C.Structure):
    _fields_ = [("rank", C.c_uint32), ("_pad", C.c_uint32), ("r_unclamped", C.c_double),
                ("H_mean", C.c_double), ("T_com", C.c_double)]


class _KernelStat(C.Structure):
    _fields_ = [("kernel", C.c_char_p), ("launches", C.c_uint64), ("total_ms", C.c_double),
                ("bytes", C.c_double), ("flops", C.c_double), ("event_overhead_ms", C.c_double)]


ENTROPY_RESULT_BYTES = C.sizeof(_EntropyResult)

_lib: Optional[C.CDLL] = None


def load_library() -> C.CDLL:
    """Loads the in-tree ``libedgc.so``; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(path)
    u64, u32, vp, i32 = C.c_uint64, C.c_uint32, C.c_void_p, C.c_int
    L.edgc_create.restype = i32
    L.edgc_create.argtypes = [C.POINTER(vp), i32, u32, u32, u64, u64]
    L.edgc_destroy.restype = i32
    L.edgc_destroy.argtypes = [vp]
    L.edgc_last_error.restype = C.c_char_p
    L.edgc_last_error.argtypes = [vp]
    L.edgc_profile_begin.restype = i32
    L.edgc_profile_begin.argtypes = [vp, u32]
    L.edgc_profile_end.restype = i32
    L.edgc_profile_end.argtypes = [vp, C.POINTER(_KernelStat), u32, C.POINTER(u32)]
    L.edgc_entropy_estimate.restype = i32
    L.edgc_entropy_estimate.argtypes = [vp, vp, i32, u64, u64, u32, u64, u64, u32, vp, vp, vp, vp]
    L.edgc_entropy_estimate_noalloc.restype = i32
    L.edgc_entropy_estimate_noalloc.argtypes = [vp, vp, i32, u64, u64, u32, u64, u64, u32, vp, vp, vp, vp]
    L.edgc_entropy_estimate_batch.restype = i32
    L.edgc_entropy_estimate_batch.argtypes = [vp, C.POINTER(C.c_void_p), C.POINTER(u64), u32, i32, u64, u32,
                                              u64, u64, u32, vp, vp, vp, vp]
    L.edgc_sample_indices.restype = i32
    L.edgc_sample_indices.argtypes = [vp, u64, u64, u32, u64, u64, vp, u64, C.POINTER(u64), vp]
    L.edgc_select_rank.restype = i32
    L.edgc_select_rank.argtypes = [C.POINTER(_RankState), vp, u32, u64, C.POINTER(_RankParams),
                                   C.POINTER(_RankDecision)]
    L.edgc_rank_bounds.restype = i32
    L.edgc_rank_bounds.argtypes = [C.POINTER(_RankCost), u32, C.c_double, C.c_double, C.c_double,
                                   C.POINTER(_RankBounds), C.POINTER(C.c_double)]
    L.edgc_fit_eta.restype = i32
    L.edgc_fit_eta.argtypes = [C.POINTER(u32), C.POINTER(C.c_double), u32, C.POINTER(C.c_double),
                               C.POINTER(C.c_double)]
    L.edgc_stage_ranks.restype = i32
    L.edgc_stage_ranks.argtypes = [u32, C.c_double, C.c_double, u32, u32, C.POINTER(u32), u32, u32,
                                   C.POINTER(u32), C.POINTER(C.c_double)]
    L.edgc_entropy_due.restype = i32
    L.edgc_entropy_due.argtypes = [u64, u32]
    L.edgc_measure_rank_costs.restype = i32
    L.edgc_measure_rank_costs.argtypes = [vp, vp, i32, u32, u32, u64, vp, vp, u32, vp, u32, vp,
                                          C.POINTER(u32), u32, u32, i32, C.POINTER(_RankCost), vp]
    L.edgc_measure_device_peaks.restype = i32
    L.edgc_measure_device_peaks.argtypes = [vp, vp, vp, u64, u32, C.POINTER(_DevicePeaks), vp]
    L.edgc_tensor_bypassed.restype = i32
    L.edgc_tensor_bypassed.argtypes = [u32, u32, u32]
    L.edgc_reserve_batch.restype = i32
    L.edgc_reserve_batch.argtypes = [vp, C.POINTER(u32), C.POINTER(u32), u32]
    L.edgc_compress_batch.restype = i32
    L.edgc_compress_batch.argtypes = [vp, C.POINTER(_Tensor), u32, i32, u32, u32, vp]
    L.edgc_decompress_batch.restype = i32
    L.edgc_decompress_batch.argtypes = [vp, C.POINTER(_Tensor), u32, i32, u32, vp]
    L.edgc_compress_p_batch.restype = i32
    L.edgc_compress_p_batch.argtypes = [vp, C.POINTER(_Tensor), u32, i32, u32, vp]
    L.edgc_compress_q_batch.restype = i32
    L.edgc_compress_q_batch.argtypes = [vp, C.POINTER(_Tensor), u32, i32, u32, vp]
    L.edgc_residual_materialize_batch.restype = i32
    L.edgc_residual_materialize_batch.argtypes = [vp, C.POINTER(_Tensor), u32, i32, u32, vp]
    L.edgc_init_q.restype = i32
    L.edgc_init_q.argtypes = [vp, vp, u32, u32, u32, u32, u64, vp]
    L.edgc_compress.restype = i32
    L.edgc_compress.argtypes = [vp, vp, i32, u32, u32, u64, vp, i32, vp, u32, vp, u32, u32, u32, vp]
    L.edgc_decompress.restype = i32
    L.edgc_decompress.argtypes = [vp, vp, u32, vp, u32, u32, u32, u32, vp, vp, i32, u64, vp]
    _lib = L
    return L


class _DevicePeaks(C.Structure):
    _fields_ = [("copy_gbs", C.c_double), ("read_gbs", C.c_double), ("mfma_bf16_tflops", C.c_double),
                ("bytes", C.c_uint64), ("write_gbs", C.c_double)]


class _Tensor(C.Structure):
    _fields_ = [("grad", C.c_void_p), ("grad_out", C.c_void_p), ("residual", C.c_void_p),
                ("Q", C.c_void_p), ("P", C.c_void_p), ("ld", C.c_uint64), ("ld_out", C.c_uint64),
                ("m", C.c_uint32), ("n", C.c_uint32), ("ldq", C.c_uint32), ("ldp", C.c_uint32),
                ("residual_is_zero", C.c_int32), ("deferred", C.c_uint32)]


@dataclass
class Tensor:
    """One entry of a batch: torch CUDA tensors (``residual``, ``Q``, ``P`` may be None for a
    tensor that is sent as it stands; 1-D gradients are taken as one row)."""
    grad: object
    grad_out: object
    residual: object = None
    Q: object = None
    P: object = None
    residual_is_zero: bool = False


class _RankCost(C.Structure):
    _fields_ = [("rank", C.c_uint32), ("_pad", C.c_uint32), ("t_compress", C.c_double),
                ("t_decompress", C.c_double), ("bytes_compressed", C.c_double)]


class _RankBounds(C.Structure):
    _fields_ = [("r_max", C.c_uint32), ("r_min", C.c_uint32), ("t_uncompressed", C.c_double)]


@dataclass
class RankCost:
    rank: int
    t_compress: float
    t_decompress: float
    bytes_compressed: float


@dataclass
class RankBounds:
    r_max: int
    r_min: int
    t_uncompressed: float
    t_com: List[float]


@dataclass
class EntropyResult:
    H_bits: float
    h_diff_nats: float
    lo: float
    hi: float
    n_sampled: int
    n_nonfinite: int
    status: int

    @staticmethod
    def from_buffer(buf) -> "EntropyResult":
        """Decode the raw result struct (e.g. a pinned uint8 tensor's bytes)."""
        r = _EntropyResult.from_buffer_copy(bytes(buf))
        return EntropyResult(r.H_bits, r.h_diff_nats, r.lo, r.hi, int(r.n_sampled),
                             int(r.n_nonfinite), int(r.status))


@dataclass
class RankParams:
    m: int
    n: int
    r_min: int
    r_max: int
    step_limit: int = 8
    allowed: Optional[Sequence[int]] = None
    eta: float = 0.0
    total_iters: int = 0
    min_warmup_frac: float = 0.10
    r_ref: int = 0


@dataclass
class RankState:
    have_ref: int = 0
    compressing: int = 0
    H_ref: float = 0.0
    r_prev: float = 0.0
    iters_seen: int = 0


@dataclass
class RankDecision:
    rank: int
    r_unclamped: float
    H_mean: float
    T_com: float


def select_rank(state: RankState, H_window: Sequence[float], iters_in_window: int,
                prm: RankParams) -> RankDecision:
    """edgc_select_rank: host-only; mutates ``state``."""
    L = load_library()
    H = (C.c_double * max(len(H_window), 1))(*[float(h) for h in H_window])
    p = _RankParams(prm.m, prm.n, prm.r_min, prm.r_max, prm.step_limit, None, 0, prm.eta,
                    prm.total_iters, prm.min_warmup_frac, prm.r_ref)
    keep = None
    if prm.allowed:
        keep = (C.c_uint32 * len(prm.allowed))(*prm.allowed)
        p.allowed = C.cast(keep, C.POINTER(C.c_uint32))
        p.n_allowed = len(prm.allowed)
    st = _RankState(state.have_ref, state.compressing, state.H_ref, state.r_prev, state.iters_seen)
    dec = _RankDecision()
    rc = L.edgc_select_rank(C.byref(st), C.cast(H, C.c_void_p), len(H_window), iters_in_window,
                            C.byref(p), C.byref(dec))
    if rc != OK:
        raise EdgcError(rc, "edgc_select_rank")
    state.have_ref, state.compressing = st.have_ref, st.compressing
    state.H_ref, state.r_prev, state.iters_seen = st.H_ref, st.r_prev, int(st.iters_seen)
    return RankDecision(int(dec.rank), dec.r_unclamped, dec.H_mean, dec.T_com)


def rank_bounds(costs: Sequence[RankCost], bytes_original: float, bandwidth: float,
                r_min_divisor: float = 4.0) -> RankBounds:
    """edgc_rank_bounds: host-only."""
    L = load_library()
    arr = (_RankCost * max(len(costs), 1))()
    for i, c in enumerate(costs):
        arr[i] = _RankCost(c.rank, 0, c.t_compress, c.t_decompress, c.bytes_compressed)
    out = _RankBounds()
    t = (C.c_double * max(len(costs), 1))()
    rc = L.edgc_rank_bounds(arr, len(costs), bytes_original, bandwidth, r_min_divisor, C.byref(out), t)
    if rc != OK:
        raise EdgcError(rc, "edgc_rank_bounds")
    return RankBounds(int(out.r_max), int(out.r_min), out.t_uncompressed, list(t)[:len(costs)])


def fit_eta(ranks: Sequence[int], t_com: Sequence[float]):
    """edgc_fit_eta: host-only.  Returns (eta, MAPE in percent)."""
    L = load_library()
    n = len(ranks)
    r = (C.c_uint32 * max(n, 1))(*[int(x) for x in ranks])
    t = (C.c_double * max(n, 1))(*[float(x) for x in t_com][:n])
    eta, mape = C.c_double(0), C.c_double(0)
    rc = L.edgc_fit_eta(r, t, n if len(t_com) == n else 0, C.byref(eta), C.byref(mape))
    if rc != OK:
        raise EdgcError(rc, "edgc_fit_eta")
    return eta.value, mape.value


def stage_ranks(r_stage1: int, t_microback: float, eta: float, r_min: int, r_max: int, n_stages: int,
                allowed: Optional[Sequence[int]] = None):
    """edgc_stage_ranks: host-only.  Returns (ranks per stage, predicted T_com per stage)."""
    L = load_library()
    ranks = (C.c_uint32 * max(n_stages, 1))()
    t = (C.c_double * max(n_stages, 1))()
    al = (C.c_uint32 * len(allowed))(*allowed) if allowed else None
    rc = L.edgc_stage_ranks(r_stage1, t_microback, eta, r_min, r_max, al, len(allowed) if allowed else 0,
                            n_stages, ranks, t)
    if rc != OK:
        raise EdgcError(rc, "edgc_stage_ranks")
    return [int(x) for x in ranks][:n_stages], list(t)[:n_stages]


def entropy_due(iter_in_window: int, period: int) -> bool:
    """edgc_entropy_due: host-only."""
    rc = load_library().edgc_entropy_due(iter_in_window, period)
    if rc < 0:
        raise EdgcError(rc, "edgc_entropy_due")
    return bool(rc)


def tensor_bypassed(m: int, n: int, r: int) -> bool:
    """edgc_tensor_bypassed: True when an m x n tensor is sent as it stands at rank r."""
    rc = load_library().edgc_tensor_bypassed(m, n, r)
    if rc < 0:
        raise EdgcError(rc, "edgc_tensor_bypassed")
    return bool(rc)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("gradient tensors must be float32 or bfloat16")


def _stream_handle(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


class PreparedBatch:
    """The descriptor array of a list of :class:`Tensor`, built once.  The batched calls take it in
    place of the list; only the two per-call flags are written again (``residual_is_zero`` from the
    Tensor objects, ``deferred`` from the call).  Pointers, shapes and leading dimensions are those
    the tensors had when it was built: build a new one after any of them changes."""

    def __init__(self, tensors: Sequence[Tensor]):
        self.tensors = list(tensors)
        self.arr, self.code = Context._marshal(self.tensors)

    def __len__(self):
        return len(self.tensors)

    def refresh(self, deferred: bool):
        d = 1 if deferred else 0
        for i, t in enumerate(self.tensors):
            a = self.arr[i]
            a.residual_is_zero = 1 if t.residual_is_zero else 0
            a.deferred = d
        return self.arr, self.code


class Context:
    """Owns an ``edgc_ctx``.  Methods take torch CUDA tensors (device memory only) and
    enqueue on ``stream`` (default: torch's current stream); nothing synchronises."""

    def __init__(self, device: int = 0, max_bins: int = 65536, max_rank: int = 128,
                 max_rows: int = 20480, max_cols: int = 20480):
        self._L = load_library()
        h = C.c_void_p()
        rc = self._L.edgc_create(C.byref(h), device, max_bins, max_rank, max_rows, max_cols)
        if rc != OK:
            raise EdgcError(rc, "edgc_create")
        self._h = h
        self.device = device

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._L.edgc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, what: str) -> None:
        if rc != OK:
            msg = self._L.edgc_last_error(self._h)
            raise EdgcError(rc, what, msg.decode() if msg else "")

    # -- per-kernel event timing ---------------------------------------------
    def profile_begin(self, max_launches: int = 4096) -> None:
        self._check(self._L.edgc_profile_begin(self._h, max_launches), "edgc_profile_begin")

    def profile_end(self) -> dict:
        """Stops the timing; returns {kernel: dict(launches, total_ms, bytes, flops)}."""
        cap = 32
        arr = (_KernelStat * cap)()
        n = C.c_uint32(0)
        self._check(self._L.edgc_profile_end(self._h, arr, cap, C.byref(n)), "edgc_profile_end")
        return {arr[i].kernel.decode(): dict(launches=int(arr[i].launches), total_ms=arr[i].total_ms,
                                             bytes=arr[i].bytes, flops=arr[i].flops,
                                             event_overhead_ms=arr[i].event_overhead_ms)
                for i in range(min(cap, n.value))}

    # -- entropy -----------------------------------------------------------
    def entropy_estimate_noalloc(self, grad, stride: int, chunk: int, seed: int, step: int, bins: int,
                                 out_pinned, value_range=None, counts_out=None, stream=None) -> None:
        """edgc_entropy_estimate_noalloc: the estimate on the library's file-scope scratch array
        (bins <= 65536); ``out_pinned`` as for :meth:`entropy_estimate_async`."""
        rng = None
        if value_range is not None:
            rng = (C.c_float * 2)(float(value_range[0]), float(value_range[1]))
        rc = self._L.edgc_entropy_estimate_noalloc(
            self._h, grad.data_ptr(), _dtype_code(grad), grad.numel(), stride, chunk, seed, step, bins,
            C.cast(rng, C.c_void_p) if rng is not None else None, out_pinned.data_ptr(),
            counts_out.data_ptr() if counts_out is not None else None, _stream_handle(stream))
        self._check(rc, "edgc_entropy_estimate_noalloc")

    def entropy_estimate_async(self, grad, stride: int, chunk: int, seed: int, step: int, bins: int,
                               out_pinned, value_range=None, counts_out=None, stream=None) -> None:
        """edgc_entropy_estimate, or edgc_entropy_estimate_batch when ``grad`` is a list of tensors
        (one estimate over the union of their samples).  ``out_pinned``: pinned uint8 CPU tensor
        of ENTROPY_RESULT_BYTES bytes, valid after the stream is synchronised."""
        rng = None
        if value_range is not None:
            rng = (C.c_float * 2)(float(value_range[0]), float(value_range[1]))
        if isinstance(grad, (list, tuple)):
            k = len(grad)
            ptrs = (C.c_void_p * max(k, 1))(*[g.data_ptr() for g in grad])
            sizes = (C.c_uint64 * max(k, 1))(*[g.numel() for g in grad])
            codes = {_dtype_code(g) for g in grad}
            if len(codes) > 1:
                raise TypeError("all buffers of one estimate must have one dtype")
            rc = self._L.edgc_entropy_estimate_batch(
                self._h, ptrs, sizes, k, codes.pop() if codes else F32, stride, chunk, seed, step, bins,
                C.cast(rng, C.c_void_p) if rng is not None else None, out_pinned.data_ptr(),
                counts_out.data_ptr() if counts_out is not None else None, _stream_handle(stream))
            self._check(rc, "edgc_entropy_estimate_batch")
            return
        rc = self._L.edgc_entropy_estimate(
            self._h, grad.data_ptr(), _dtype_code(grad), grad.numel(), stride, chunk, seed, step, bins,
            C.cast(rng, C.c_void_p) if rng is not None else None, out_pinned.data_ptr(),
            counts_out.data_ptr() if counts_out is not None else None, _stream_handle(stream))
        self._check(rc, "edgc_entropy_estimate")

    def entropy_estimate(self, grad, stride: int, chunk: int, seed: int, step: int, bins: int,
                         value_range=None, counts_out=None, stream=None) -> EntropyResult:
        """Blocking convenience wrapper: runs the estimate and synchronises the stream."""
        import torch
        out = torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True)
        self.entropy_estimate_async(grad, stride, chunk, seed, step, bins, out, value_range,
                                    counts_out, stream)
        (stream if stream is not None else torch.cuda.current_stream()).synchronize()
        return EntropyResult.from_buffer(out.numpy().tobytes())

    def sample_indices(self, n_elems: int, stride: int, chunk: int, seed: int, step: int,
                       idx_out=None, stream=None) -> int:
        """edgc_sample_indices.  Returns the sample size; fills ``idx_out`` (int64 CUDA tensor)."""
        n = C.c_uint64(0)
        rc = self._L.edgc_sample_indices(
            self._h, n_elems, stride, chunk, seed, step,
            idx_out.data_ptr() if idx_out is not None else None,
            idx_out.numel() if idx_out is not None else 0, C.byref(n), _stream_handle(stream))
        self._check(rc, "edgc_sample_indices")
        return int(n.value)

    # -- compressor --------------------------------------------------------
    def init_q(self, Q, col_begin: int, col_end: int, seed: int, stream=None) -> None:
        assert Q.dim() == 2 and Q.is_contiguous()
        rc = self._L.edgc_init_q(self._h, Q.data_ptr(), Q.shape[0], Q.shape[1], col_begin, col_end,
                                 seed, _stream_handle(stream))
        self._check(rc, "edgc_init_q")

    def compress(self, grad, residual, residual_is_zero: bool, Q, P, r: int, power_iters: int = 1,
                 stream=None) -> None:
        """edgc_compress.  grad (m, n) fp32/bf16 (row stride = grad.stride(0)); residual (m, n)
        fp32 contiguous; Q (n, ldq) and P (m, ldp) fp32 contiguous with ldq, ldp >= r."""
        m, n = grad.shape
        rc = self._L.edgc_compress(
            self._h, grad.data_ptr(), _dtype_code(grad), m, n, grad.stride(0), residual.data_ptr(),
            1 if residual_is_zero else 0, Q.data_ptr(), Q.shape[1], P.data_ptr(), P.shape[1], r,
            power_iters, _stream_handle(stream))
        self._check(rc, "edgc_compress")

    def decompress(self, P, Q, r: int, residual, grad_out, stream=None) -> None:
        """edgc_decompress.  residual (m, n) holds D on entry and E_new on return."""
        m, n = grad_out.shape
        rc = self._L.edgc_decompress(
            self._h, P.data_ptr(), P.shape[1], Q.data_ptr(), Q.shape[1], m, n, r, residual.data_ptr(),
            grad_out.data_ptr(), _dtype_code(grad_out), grad_out.stride(0), _stream_handle(stream))
        self._check(rc, "edgc_decompress")

    def measure_rank_costs(self, grad, residual, Q, P, grad_out, ranks: Sequence[int], reps: int = 5,
                           stream=None, deferred: bool = False) -> List[RankCost]:
        """edgc_measure_rank_costs: times compress and decompress at each rank on these buffers
        (all overwritten except grad); synchronises the stream.  ``deferred``: time the deferred
        form of the residual."""
        m, n = grad.shape
        rk = (C.c_uint32 * max(len(ranks), 1))(*[int(r) for r in ranks])
        out = (_RankCost * max(len(ranks), 1))()
        rc = self._L.edgc_measure_rank_costs(
            self._h, grad.data_ptr(), _dtype_code(grad), m, n, grad.stride(0), residual.data_ptr(),
            Q.data_ptr(), Q.shape[1], P.data_ptr(), P.shape[1], grad_out.data_ptr(), rk, len(ranks),
            reps, 1 if deferred else 0, out, _stream_handle(stream))
        self._check(rc, "edgc_measure_rank_costs")
        return [RankCost(int(c.rank), c.t_compress, c.t_decompress, c.bytes_compressed)
                for c in list(out)[:len(ranks)]]

    def measure_device_peaks(self, buf_a, buf_b, reps: int = 10, stream=None) -> dict:
        """edgc_measure_device_peaks: what a plain copy, a plain read and a bf16 MFMA loop reach on
        this device; buf_a is read, buf_b overwritten (two tensors of equal size in bytes);
        synchronises the stream."""
        nbytes = buf_a.numel() * buf_a.element_size()
        if nbytes != buf_b.numel() * buf_b.element_size():
            raise ValueError("the two buffers must have the same size in bytes")
        out = _DevicePeaks()
        rc = self._L.edgc_measure_device_peaks(self._h, buf_a.data_ptr(), buf_b.data_ptr(), nbytes, reps,
                                               C.byref(out), _stream_handle(stream))
        self._check(rc, "edgc_measure_device_peaks")
        return {"copy_gbs": out.copy_gbs, "read_gbs": out.read_gbs,
                "mfma_bf16_tflops": out.mfma_bf16_tflops, "bytes": int(out.bytes),
                "write_gbs": out.write_gbs}

    # -- batched calls -----------------------------------------------------
    def reserve_batch(self, shapes: Sequence[Sequence[int]]) -> None:
        """edgc_reserve_batch: position i of later batches holds at most shapes[i] = (rows, cols)."""
        n = len(shapes)
        rows = (C.c_uint32 * max(n, 1))(*[int(s[0]) for s in shapes])
        cols = (C.c_uint32 * max(n, 1))(*[int(s[1]) for s in shapes])
        self._check(self._L.edgc_reserve_batch(self._h, rows, cols, n), "edgc_reserve_batch")

    @staticmethod
    def _marshal(tensors, deferred: bool = False):
        if isinstance(tensors, PreparedBatch):
            return tensors.refresh(deferred)
        arr = (_Tensor * max(len(tensors), 1))()
        code = None
        for i, t in enumerate(tensors):
            g = t.grad if t.grad is not None else t.grad_out
            m, n = (1, g.numel()) if g.dim() == 1 else g.shape
            ld = lambda x: (x.stride(0) if x.dim() == 2 else x.numel()) if x is not None else 0
            ptr = lambda x: x.data_ptr() if x is not None else None
            arr[i] = _Tensor(ptr(t.grad), ptr(t.grad_out), ptr(t.residual), ptr(t.Q), ptr(t.P),
                             ld(t.grad), ld(t.grad_out), m, n,
                             t.Q.shape[1] if t.Q is not None else 0,
                             t.P.shape[1] if t.P is not None else 0,
                             1 if t.residual_is_zero else 0, 1 if deferred else 0)
            c = _dtype_code(g)
            if code is not None and c != code:
                raise TypeError("all gradients of a batch must have one dtype")
            code = c
        return arr, (code if code is not None else F32)

    def compress_batch(self, tensors: Sequence[Tensor], r: int, power_iters: int = 1, stream=None,
                       deferred: bool = False) -> None:
        """edgc_compress_batch over a list of :class:`Tensor`; ``deferred``: the residual buffers
        hold D of the previous step and P, Q its factors (edgc_tensor.deferred of every entry)."""
        arr, code = self._marshal(tensors, deferred)
        rc = self._L.edgc_compress_batch(self._h, arr, len(tensors), code, r, power_iters,
                                         _stream_handle(stream))
        self._check(rc, "edgc_compress_batch")

    def compress_p_batch(self, tensors: Sequence[Tensor], r: int, stream=None, deferred: bool = False) -> None:
        """edgc_compress_p_batch: error-feedback add and P-pass; P is left un-orthonormalised."""
        arr, code = self._marshal(tensors, deferred)
        rc = self._L.edgc_compress_p_batch(self._h, arr, len(tensors), code, r, _stream_handle(stream))
        self._check(rc, "edgc_compress_p_batch")

    def compress_q_batch(self, tensors: Sequence[Tensor], r: int, stream=None) -> None:
        """edgc_compress_q_batch: orthonormalise P as it stands, then the Q-pass."""
        arr, code = self._marshal(tensors)
        rc = self._L.edgc_compress_q_batch(self._h, arr, len(tensors), code, r, _stream_handle(stream))
        self._check(rc, "edgc_compress_q_batch")

    def decompress_batch(self, tensors: Sequence[Tensor], r: int, stream=None, deferred: bool = False) -> None:
        """edgc_decompress_batch over a list of :class:`Tensor`; ``deferred``: only the
        reconstruction is written and the residual buffers keep D."""
        arr, code = self._marshal(tensors, deferred)
        rc = self._L.edgc_decompress_batch(self._h, arr, len(tensors), code, r, _stream_handle(stream))
        self._check(rc, "edgc_decompress_batch")

    def residual_materialize_batch(self, tensors: Sequence[Tensor], r: int, stream=None) -> None:
        """edgc_residual_materialize_batch: residual <- residual - round(P Q^T)."""
        arr, code = self._marshal(tensors)
        rc = self._L.edgc_residual_materialize_batch(self._h, arr, len(tensors), code, r,
                                                     _stream_handle(stream))
        self._check(rc, "edgc_residual_materialize_batch")
