"""ctypes wrapper over the C oracle (``edgc_oracle.c``) -- test infrastructure.

Argument marshalling only; every number is produced by the C code.  bf16
tensors travel as ``numpy.uint16`` arrays holding the raw bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
OK, EINVAL, ENOMEM, ENONFINITE = 0, -1, -2, -5


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


class _EntropyResult(C.Structure):
    _fields_ = [("H_bits", C.c_double), ("h_diff_nats", C.c_double), ("lo", C.c_float),
                ("hi", C.c_float), ("n_sampled", C.c_uint64), ("n_nonfinite", C.c_uint64)]


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


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build(force=True)
        L = C.CDLL(path)
        u64, u32, dbl, vp = C.c_uint64, C.c_uint32, C.c_double, C.c_void_p
        L.oracle_mix64.restype = u64
        L.oracle_mix64.argtypes = [u64, u64]
        L.oracle_sample_slot.restype = u64
        L.oracle_sample_slot.argtypes = [u64, u64, u64]
        L.oracle_sample_indices.restype = u64
        L.oracle_sample_indices.argtypes = [u64, u64, u32, u64, u64, vp, u64]
        L.oracle_entropy.restype = C.c_int
        L.oracle_entropy.argtypes = [vp, C.c_int, u64, u64, u32, u64, u64, u32, vp,
                                     C.POINTER(_EntropyResult), vp]
        L.oracle_mp_cdf.restype = dbl
        L.oracle_mp_cdf.argtypes = [dbl, u32, u32]
        L.oracle_mp_quantile.restype = dbl
        L.oracle_mp_quantile.argtypes = [dbl, u32, u32]
        L.oracle_g_table.restype = C.c_int64
        L.oracle_g_table.argtypes = [u32, u32, vp]
        L.oracle_select_rank.restype = C.c_int
        L.oracle_select_rank.argtypes = [C.POINTER(_RankState), vp, u32, u64,
                                         C.POINTER(_RankParams), C.POINTER(_RankDecision)]
        L.oracle_init_q.restype = None
        L.oracle_init_q.argtypes = [vp, u32, u32, u32, u32, u64]
        L.oracle_compress.restype = C.c_int
        L.oracle_compress.argtypes = [vp, C.c_int, u32, u32, u64, vp, C.c_int, vp, u32, vp, u32,
                                      u32, u32]
        L.oracle_decompress.restype = C.c_int
        L.oracle_decompress.argtypes = [vp, u32, vp, u32, u32, u32, u32, vp, vp, C.c_int, u64]
        L.oracle_contract_p.restype = C.c_int
        L.oracle_contract_p.argtypes = [vp, u32, u32, vp, u32, u32, C.c_int, vp, u32]
        L.oracle_contract_q.restype = C.c_int
        L.oracle_contract_q.argtypes = [vp, u32, u32, vp, u32, u32, C.c_int, vp, u32]
        L.oracle_orthonormalise.restype = C.c_int
        L.oracle_orthonormalise.argtypes = [vp, u32, u32, u32]
        L.oracle_reconstruct_one.restype = dbl
        L.oracle_reconstruct_one.argtypes = [vp, u32, vp, u32, u32, u32, u32, C.c_int]
        L.oracle_bf16_to_f32.restype = C.c_float
        L.oracle_bf16_to_f32.argtypes = [C.c_uint16]
        L.oracle_f32_to_bf16.restype = C.c_uint16
        L.oracle_f32_to_bf16.argtypes = [C.c_float]
        L.oracle_num_threads.restype = C.c_int
        L.oracle_set_num_threads.restype = None
        L.oracle_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _check_grad(grad: np.ndarray) -> int:
    if grad.dtype == np.float32:
        return F32
    if grad.dtype == np.uint16:
        return BF16
    raise TypeError("gradient must be float32 or uint16 (raw bf16 bits)")


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the oracle's loops over independent outputs use from now on (no effect on results)."""
    lib().oracle_set_num_threads(int(n))


def mix64(seed: int, ctr: int) -> int:
    return int(lib().oracle_mix64(seed, ctr))


def sample_slot(seed: int, step: int, stride: int) -> int:
    return int(lib().oracle_sample_slot(seed, step, stride))


def sample_indices(n: int, stride: int, chunk: int, seed: int, step: int) -> np.ndarray:
    cnt = int(lib().oracle_sample_indices(n, stride, chunk, seed, step, None, 0))
    idx = np.empty(cnt, dtype=np.uint64)
    got = int(lib().oracle_sample_indices(n, stride, chunk, seed, step, _ptr(idx), cnt))
    assert got == cnt
    return idx


@dataclass
class EntropyResult:
    H_bits: float
    h_diff_nats: float
    lo: float
    hi: float
    n_sampled: int
    n_nonfinite: int
    counts: np.ndarray


def entropy(grad: np.ndarray, stride: int, chunk: int, seed: int, step: int, bins: int,
            value_range: Optional[Sequence[float]] = None) -> EntropyResult:
    """Histogram entropy of the sampled subset (Sec. IV-B, Eq. (1))."""
    g = np.ascontiguousarray(grad).reshape(-1)
    dt = _check_grad(g)
    res = _EntropyResult()
    counts = np.zeros(max(bins, 1), dtype=np.uint64)
    rng = None
    if value_range is not None:
        rng = np.asarray(value_range, dtype=np.float32)
    rc = lib().oracle_entropy(_ptr(g), dt, g.size, stride, chunk, seed, step, bins,
                              _ptr(rng) if rng is not None else None, C.byref(res), _ptr(counts))
    if rc != OK:
        raise OracleError(rc, "oracle_entropy")
    return EntropyResult(res.H_bits, res.h_diff_nats, res.lo, res.hi, int(res.n_sampled),
                         int(res.n_nonfinite), counts[:bins])


def mp_cdf(lam: float, m: int, n: int) -> float:
    return float(lib().oracle_mp_cdf(lam, m, n))


def mp_quantile(p: float, m: int, n: int) -> float:
    return float(lib().oracle_mp_quantile(p, m, n))


def g_table(m: int, n: int) -> np.ndarray:
    mm = min(m, n)
    g = np.empty(mm + 1, dtype=np.float64)
    got = int(lib().oracle_g_table(m, n, _ptr(g)))
    assert got == mm
    return g


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
    """Window rule: Theorem 3 + Sec. IV-D-2 warm-up + Algorithm 1.  Mutates ``state``."""
    H = np.ascontiguousarray(np.asarray(H_window, dtype=np.float64))
    allowed = None
    p = _RankParams(prm.m, prm.n, prm.r_min, prm.r_max, prm.step_limit, None, 0, prm.eta,
                    prm.total_iters, prm.min_warmup_frac, prm.r_ref)
    if prm.allowed:
        allowed = (C.c_uint32 * len(prm.allowed))(*prm.allowed)
        p.allowed = C.cast(allowed, C.POINTER(C.c_uint32))
        p.n_allowed = len(prm.allowed)
    st = _RankState(state.have_ref, state.compressing, state.H_ref, state.r_prev, state.iters_seen)
    dec = _RankDecision()
    rc = lib().oracle_select_rank(C.byref(st), _ptr(H) if H.size else None, H.size,
                                  iters_in_window, C.byref(p), C.byref(dec))
    if rc != OK:
        raise OracleError(rc, "oracle_select_rank")
    state.have_ref, state.compressing = st.have_ref, st.compressing
    state.H_ref, state.r_prev, state.iters_seen = st.H_ref, st.r_prev, int(st.iters_seen)
    return RankDecision(int(dec.rank), dec.r_unclamped, dec.H_mean, dec.T_com)


def init_q(Q: np.ndarray, col_begin: int, col_end: int, seed: int) -> None:
    """Fill columns [col_begin, col_end) of the fp32 (n x ld) array Q with seeded N(0,1)."""
    assert Q.dtype == np.float32 and Q.ndim == 2 and Q.flags.c_contiguous
    lib().oracle_init_q(_ptr(Q), Q.shape[0], Q.shape[1], col_begin, col_end, seed)


def compress(grad: np.ndarray, residual: Optional[np.ndarray], Q: np.ndarray, r: int,
             power_iters: int = 1):
    """One compression step.  Returns (P_hat, Q_new, Delta); inputs are not modified.

    grad: (m, n) float32 or uint16 (bf16 bits); residual: (m, n) float32 or None (zero);
    Q: (n, >=r) float32 warm start (only the first r columns are used).
    """
    g = np.ascontiguousarray(grad)
    dt = _check_grad(g)
    m, n = g.shape
    zero = residual is None
    D = np.empty((m, n), dtype=np.float32) if zero else np.array(residual, dtype=np.float32,
                                                               order="C", copy=True)
    Qw = np.array(Q[:, :r], dtype=np.float32, order="C", copy=True)
    P = np.zeros((m, r), dtype=np.float32)
    rc = lib().oracle_compress(_ptr(g), dt, m, n, n, _ptr(D), int(zero), _ptr(Qw), r, _ptr(P), r,
                               r, power_iters)
    if rc != OK:
        raise OracleError(rc, "oracle_compress")
    return P, Qw, D


def decompress(P: np.ndarray, Q: np.ndarray, delta: np.ndarray, dtype: int):
    """M_hat = P Q^T rounded to ``dtype``; returns (out, E_new).  Inputs are not modified."""
    P = np.ascontiguousarray(P, dtype=np.float32)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    m, r = P.shape
    n = Q.shape[0]
    assert Q.shape[1] == r and delta.shape == (m, n)
    E = np.array(delta, dtype=np.float32, order="C", copy=True)
    out = np.empty((m, n), dtype=np.uint16 if dtype == BF16 else np.float32)
    rc = lib().oracle_decompress(_ptr(P), r, _ptr(Q), r, m, n, r, _ptr(E), _ptr(out), dtype, n)
    if rc != OK:
        raise OracleError(rc, "oracle_decompress")
    return out, E


def contract_p(D: np.ndarray, Q: np.ndarray, dtype: int) -> np.ndarray:
    """P = D Q as the compress step forms it (D: rows x n fp32, e.g. gathered rows; Q: n x r)."""
    D = np.ascontiguousarray(D, dtype=np.float32)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    m, n = D.shape
    r = Q.shape[1]
    assert Q.shape[0] == n
    P = np.zeros((m, r), dtype=np.float32)
    rc = lib().oracle_contract_p(_ptr(D), m, n, _ptr(Q), r, r, dtype, _ptr(P), r)
    if rc != OK:
        raise OracleError(rc, "oracle_contract_p")
    return P


def contract_q(D: np.ndarray, P: np.ndarray, dtype: int) -> np.ndarray:
    """Q = D^T P^ as the compress step forms it (D: m x cols fp32, e.g. gathered columns; P: m x r)."""
    D = np.ascontiguousarray(D, dtype=np.float32)
    P = np.ascontiguousarray(P, dtype=np.float32)
    m, n = D.shape
    r = P.shape[1]
    assert P.shape[0] == m
    Q = np.zeros((n, r), dtype=np.float32)
    rc = lib().oracle_contract_q(_ptr(D), m, n, _ptr(P), r, r, dtype, _ptr(Q), r)
    if rc != OK:
        raise OracleError(rc, "oracle_contract_q")
    return Q


def orthonormalise(P: np.ndarray) -> np.ndarray:
    """The orthonormalisation step of compress (modified Gram-Schmidt in fp64) on a copy of P."""
    out = np.array(P, dtype=np.float32, order="C", copy=True)
    rc = lib().oracle_orthonormalise(_ptr(out), out.shape[0], out.shape[1], out.shape[1])
    if rc != OK:
        raise OracleError(rc, "oracle_orthonormalise")
    return out


def reconstruct_one(P: np.ndarray, Q: np.ndarray, i: int, j: int, dtype: int) -> float:
    P = np.ascontiguousarray(P, dtype=np.float32)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    return float(lib().oracle_reconstruct_one(_ptr(P), P.shape[1], _ptr(Q), Q.shape[1],
                                              P.shape[1], i, j, dtype))


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of raw bf16 bit patterns (uint16) to float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_scalar(x: float) -> int:
    return int(lib().oracle_f32_to_bf16(C.c_float(x)))
