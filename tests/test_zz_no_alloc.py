"""The entry point that allocates nothing (edgc_entropy_estimate_noalloc) against the entry point it
is a variant of (edgc_entropy_estimate), through the C ABI: same range, same 64-bit counts bit for
bit, entropy within 1e-5 (both evaluate it in fp64 from identical counts), on calls in a row that
share the library's file-scope scratch array, a later call with a smaller input and fewer bins than
the one before it (what the earlier call left in the array must not leak into the later result)."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from paper_2511_10333_amd import binding
from gpu_util import ctx, to_dev

pytestmark = pytest.mark.gpu


def _call(name, c, x, stride, chunk, seed, step, bins, value_range, with_counts):
    """One estimate through the raw C symbol `name`; returns (result, counts or None)."""
    L = binding.load_library()
    fn = getattr(L, name)
    out = torch.zeros(binding.ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True)
    counts = torch.full((bins,), -1, dtype=torch.int64, device="cuda") if with_counts else None
    rng = (C.c_float * 2)(*value_range) if value_range is not None else None
    torch.cuda.synchronize()
    rc = fn(c._h, x.data_ptr(), binding.BF16 if x.dtype == torch.bfloat16 else binding.F32, x.numel(), stride, chunk,
            seed, step, bins, C.cast(rng, C.c_void_p) if rng is not None else None, out.data_ptr(),
            counts.data_ptr() if counts is not None else None, int(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, L.edgc_last_error(c._h)
    torch.cuda.synchronize()
    res = edgc.EntropyResult.from_buffer(out.numpy().tobytes())
    return res, (counts.cpu().numpy() if counts is not None else None)


def _same(a, b):
    ra, ca = a
    rb, cb = b
    assert ra.status == rb.status == 0
    assert (ra.lo, ra.hi, ra.n_sampled, ra.n_nonfinite) == (rb.lo, rb.hi, rb.n_sampled, rb.n_nonfinite)
    if ca is not None:
        assert np.array_equal(ca, cb) and ca.min() >= 0
    assert abs(ra.H_bits - rb.H_bits) <= 1e-5
    if math.isinf(rb.h_diff_nats):
        assert ra.h_diff_nats == rb.h_diff_nats
    else:
        assert abs(ra.h_diff_nats - rb.h_diff_nats) <= 1e-5


# each case: (elements, dtype, stride, chunk, bins, caller range, counts to the caller)
CASES = [
    (1 << 22, "f32", 1, 64, 65536, None, True),        # every element, two LDS slices, the array's largest histogram
    (300_007, "f32", 10, 64, 256, None, False),        # smaller input, fewer bins, histogram in the array itself
    (1 << 20, "bf16", 100, 64, 4096, None, True),
    (70_001, "bf16", 1, 1, 1024, (-2e-3, 2e-3), False),
    (5000, "f32", 3, 4096, 16, None, True),
]


def test_noalloc_estimate_equals_the_context_estimate_on_calls_in_a_row():
    c = ctx(max_bins=1 << 20)
    for rep in range(2):                                # the whole sequence twice: the array is reused
        for k, (n, dt, stride, chunk, bins, rng, with_counts) in enumerate(CASES):
            x = to_dev(gen.laplace_mixture(n, seed=10 + k, dtype=dt))
            if k == 2:
                x[12345] = float("nan")                 # a skipped value: n_nonfinite = 1 on both sides
            want = _call("edgc_entropy_estimate", c, x, stride, chunk, 3, rep, bins, rng, with_counts)
            got = _call("edgc_entropy_estimate_noalloc", c, x, stride, chunk, 3, rep, bins, rng, with_counts)
            _same(got, want)
            if not with_counts:
                # the histogram stayed in the array: a second call on the same input gives the same again
                _same(_call("edgc_entropy_estimate_noalloc", c, x, stride, chunk, 3, rep, bins, rng, False), want)


def test_noalloc_estimate_limits_and_second_context():
    c = ctx(max_bins=1 << 20)
    x = to_dev(gen.gaussian(10_000, 1e-3, 5))
    L = binding.load_library()
    out = torch.zeros(binding.ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True)
    st = int(torch.cuda.current_stream().cuda_stream)
    # beyond the array's histogram: a clear error, nothing launched
    rc = L.edgc_entropy_estimate_noalloc(c._h, x.data_ptr(), binding.F32, x.numel(), 1, 64, 0, 0, 65537, None,
                                         out.data_ptr(), None, st)
    assert rc == binding.EINVAL and b"65536" in L.edgc_last_error(c._h)
    rc = L.edgc_entropy_estimate_noalloc(c._h, x.data_ptr(), binding.F32, x.numel(), 1, 64, 0, 0, 0, None,
                                         out.data_ptr(), None, st)
    assert rc == binding.EINVAL
    # a context created with a small max_bins still takes the array's limit, and a second context on
    # the same GPU shares the array with the first (calls in sequence)
    small = edgc.Context(0, max_bins=16, max_rank=4, max_rows=64, max_cols=64)
    try:
        want = _call("edgc_entropy_estimate", c, x, 1, 64, 0, 0, 2048, None, True)
        _same(_call("edgc_entropy_estimate_noalloc", small, x, 1, 64, 0, 0, 2048, None, True), want)
        _same(_call("edgc_entropy_estimate_noalloc", c, x, 1, 64, 0, 0, 2048, None, True), want)
    finally:
        small.close()
