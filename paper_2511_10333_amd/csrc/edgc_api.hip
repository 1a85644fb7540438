// C-ABI entry points of libedgc (include/edgc.h): argument checks, context and
// scratch management, and hand-off to the kernel launchers.  No computation here.
#include "edgc_internal.h"

#include <algorithm>
#include <cstdlib>
#include <new>

using namespace edgc;

namespace edgc {
const char* const kKernelNames[KID_COUNT] = {
    "k_set_range", "k_minmax", "k_hist", "k_sample_indices", "k_init_q", "k_pass_p",
    "k_reduce_gram", "k_gram_sum", "k_chol", "k_apply", "k_pass_q", "k_reduce_q", "k_decompress",
    "k_pass_p_deferred", "k_wide_hist", "k_wide_reduce"};
}

namespace {

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

template <typename T>
hipError_t dev_alloc(T** p, size_t count)
{
    *p = nullptr;
    return hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T));
}

void free_batch(edgc_ctx* ctx)
{
    for (BatchSlot& b : ctx->batch) {
        for (void* p : {static_cast<void*>(b.part), static_cast<void*>(b.gram_part),
                        static_cast<void*>(b.gram), static_cast<void*>(b.rinv), b.pt})
            if (p) (void)hipFree(p);
    }
    ctx->batch.clear();
}

void free_scratch(Scratch& s)
{
    void* ptrs[] = {s.mm_part, s.done_counter, s.part16, s.wide, s.totals, s.counts, s.range, s.result_dev,
                    s.part, s.gram_part, s.gram, s.rinv, s.pt};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    s = Scratch{};
}

}  // namespace

extern "C" int edgc_create(edgc_ctx** out, int hip_device, uint32_t max_bins, uint32_t max_rank,
                           uint64_t max_rows, uint64_t max_cols)
{
    if (!out) return EDGC_EINVAL;
    *out = nullptr;
    if (max_bins == 0 || max_bins > (1u << 24) || max_rank == 0 || max_rank > 128 || max_rows == 0 ||
        max_cols == 0 || max_rows > kMaxDim || max_cols > kMaxDim)
        return EDGC_EINVAL;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || hip_device < 0 || hip_device >= ndev) return EDGC_EHIP;
    if (hipSetDevice(hip_device) != hipSuccess) return EDGC_EHIP;

    edgc_ctx* ctx = new (std::nothrow) edgc_ctx();
    if (!ctx) return EDGC_ENOMEM;
    ctx->device = hip_device;
    ctx->max_bins = max_bins;
    ctx->max_rank = max_rank;
    ctx->max_rows = max_rows;
    ctx->max_cols = max_cols;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, hip_device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->num_cu = prop.multiProcessorCount;

    // developer knobs for launch-shape sweeps (environment, read once per context)
    if (const char* e = getenv("EDGC_TUNE_P")) ctx->tune_p = std::max(1, atoi(e));
    if (const char* e = getenv("EDGC_TUNE_Q")) ctx->tune_q = std::max(1, atoi(e));
    if (const char* e = getenv("EDGC_TUNE_D")) ctx->tune_d = std::max(1, atoi(e));
    if (const char* e = getenv("EDGC_TUNE_STREAM")) ctx->tune_stream = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_FULL")) ctx->tune_full = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_DFULL")) ctx->tune_dfull = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_PATTERN")) ctx->tune_pattern = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_QFULL")) ctx->tune_qfull = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_PWAVES")) ctx->tune_pwaves = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_APPLY")) ctx->tune_apply = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_EPT")) ctx->tune_ept = atoi(e);
    if (const char* e = getenv("EDGC_TUNE_PATTERN_MIN")) ctx->tune_pattern_min = atoll(e);

    Scratch& s = ctx->s;
    const uint64_t rp = (max_rank <= 32) ? 32 : (max_rank <= 64 ? 64 : 128);
    const uint64_t rows_pad = (max_rows + 63) / 64 * 64;
    s.part_elems = compress_part_elems(max_rows, max_cols, max_rank, ctx->num_cu);
    // per-block upper-triangle 16x16 Gram tiles: at most 36 tiles of 256 doubles per 64-row chunk
    s.gram_part_elems = (rows_pad / 64) * 36ull * 256ull;
    s.pt_bytes = 2ull * rp * rows_pad * 2ull;
    bool ok = true;
    ok = ok && dev_alloc(&s.mm_part, 2 * kMaxReduceBlocks) == hipSuccess;
    ok = ok && dev_alloc(&s.done_counter, 4) == hipSuccess;
    s.part16_blocks = static_cast<uint32_t>(ctx->num_cu);
    ok = ok && dev_alloc(&s.part16, static_cast<size_t>(s.part16_blocks) * 65536) == hipSuccess;
    ok = ok && dev_alloc(&s.wide, 65536) == hipSuccess;
    ok = ok && dev_alloc(&s.totals, 65536) == hipSuccess;
    ok = ok && dev_alloc(&s.counts, max_bins) == hipSuccess;
    ok = ok && hipMalloc(&s.range, 64) == hipSuccess;
    ok = ok && hipMalloc(&s.result_dev, sizeof(edgc_entropy_result)) == hipSuccess;
    ok = ok && dev_alloc(&s.part, s.part_elems) == hipSuccess;
    ok = ok && dev_alloc(&s.gram_part, s.gram_part_elems) == hipSuccess;
    ok = ok && dev_alloc(&s.gram, static_cast<size_t>(36) * 256) == hipSuccess;
    ok = ok && dev_alloc(&s.rinv, rinv_elems(max_rank)) == hipSuccess;
    ok = ok && hipMalloc(&s.pt, s.pt_bytes) == hipSuccess;
    ok = ok && hipMemset(s.done_counter, 0, 4 * sizeof(unsigned int)) == hipSuccess;
    ok = ok && hipMemset(s.wide, 0, 65536 * sizeof(unsigned long long)) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    ok = ok && prepare_entropy_kernels(ctx) == EDGC_OK && prepare_compress_kernels(ctx) == EDGC_OK;
    ok = ok && resolve_static_scratch(ctx) == EDGC_OK;
    if (!ok) {
        (void)hipGetLastError();
        free_scratch(s);
        delete ctx;
        return EDGC_ENOMEM;
    }
    *out = ctx;
    return EDGC_OK;
}

extern "C" int edgc_profile_begin(edgc_ctx* ctx, uint32_t max_launches)
{
    if (!ctx) return EDGC_EINVAL;
    if (max_launches < 16 || max_launches > (1u << 20)) return fail(ctx, EDGC_EINVAL, "max_launches out of range");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    Profiler& p = ctx->prof;
    while (p.pool.size() < 2ull * max_launches) {
        hipEvent_t e;
        EDGC_HIP_TRY(ctx, hipEventCreate(&e));
        p.pool.push_back(e);
    }
    p.next = 0;
    p.recs.clear();
    p.recs.reserve(max_launches);
    // What an event pair reads with nothing between the two records: subtracted from every
    // bracketed launch in edgc_profile_end (median of 15 pairs on the default stream).
    {
        constexpr int kPairs = 15;
        float gap[kPairs];
        EDGC_HIP_TRY(ctx, hipDeviceSynchronize());
        for (int i = 0; i < kPairs; ++i) {
            EDGC_HIP_TRY(ctx, hipEventRecord(p.pool[2 * i], nullptr));
            EDGC_HIP_TRY(ctx, hipEventRecord(p.pool[2 * i + 1], nullptr));
        }
        EDGC_HIP_TRY(ctx, hipDeviceSynchronize());
        for (int i = 0; i < kPairs; ++i)
            EDGC_HIP_TRY(ctx, hipEventElapsedTime(&gap[i], p.pool[2 * i], p.pool[2 * i + 1]));
        std::sort(gap, gap + kPairs);
        p.empty_pair_ms = gap[kPairs / 2];
    }
    p.on = true;
    return EDGC_OK;
}

extern "C" int edgc_profile_end(edgc_ctx* ctx, edgc_kernel_stat* out, uint32_t cap, uint32_t* n_out)
{
    if (!ctx) return EDGC_EINVAL;
    if (!n_out || (!out && cap)) return fail(ctx, EDGC_EINVAL, "null output");
    Profiler& p = ctx->prof;
    p.on = false;
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    EDGC_HIP_TRY(ctx, hipDeviceSynchronize());
    edgc_kernel_stat acc[KID_COUNT] = {};
    for (const ProfRec& r : p.recs) {
        float ms = 0.0f;
        EDGC_HIP_TRY(ctx, hipEventElapsedTime(&ms, r.a, r.b));
        acc[r.kid].launches += 1;
        acc[r.kid].total_ms += std::max(0.0, static_cast<double>(ms) - p.empty_pair_ms);
        acc[r.kid].event_overhead_ms = p.empty_pair_ms;
        acc[r.kid].bytes += r.bytes;
        acc[r.kid].flops += r.flops;
    }
    uint32_t n = 0;
    for (int k = 0; k < KID_COUNT; ++k) {
        if (!acc[k].launches) continue;
        if (n < cap) { out[n] = acc[k]; out[n].kernel = kKernelNames[k]; }
        ++n;
    }
    *n_out = n;
    p.recs.clear();
    p.next = 0;
    return EDGC_OK;
}

extern "C" int edgc_destroy(edgc_ctx* ctx)
{
    if (!ctx) return EDGC_EINVAL;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    for (hipEvent_t e : ctx->prof.pool) (void)hipEventDestroy(e);
    free_batch(ctx);
    free_scratch(ctx->s);
    delete ctx;
    return EDGC_OK;
}

extern "C" const char* edgc_last_error(const edgc_ctx* ctx)
{
    return ctx ? ctx->last_error.c_str() : "null context";
}

static int check_sampler_args(edgc_ctx* ctx, uint64_t stride, uint32_t chunk)
{
    if (stride == 0 || chunk == 0) return fail(ctx, EDGC_EINVAL, "stride and chunk must be >= 1");
    if (stride > (1ull << 40) || chunk > (1u << 20))
        return fail(ctx, EDGC_EINVAL, "stride > 2^40 or chunk > 2^20");
    return EDGC_OK;
}

extern "C" int edgc_entropy_estimate(edgc_ctx* ctx, const void* grad, edgc_dtype dtype,
                                     uint64_t n_elems, uint64_t stride, uint32_t chunk, uint64_t seed,
                                     uint64_t step, uint32_t bins, const float* range,
                                     edgc_entropy_result* out, uint64_t* counts_out, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!grad || !out) return fail(ctx, EDGC_EINVAL, "null grad or out");
    if (dtype != EDGC_F32 && dtype != EDGC_BF16) return fail(ctx, EDGC_EINVAL, "unknown dtype");
    if (int rc = check_sampler_args(ctx, stride, chunk)) return rc;
    if (bins == 0 || bins > ctx->max_bins) return fail(ctx, EDGC_EINVAL, "bins == 0 or bins > max_bins");
    if (range && !(range[0] <= range[1])) return fail(ctx, EDGC_EINVAL, "range needs lo <= hi");
    return edgc_entropy_estimate_batch(ctx, &grad, &n_elems, 1, dtype, stride, chunk, seed, step, bins, range,
                                       out, counts_out, hip_stream);
}

static int entropy_estimate_impl(edgc_ctx* ctx, bool static_scratch, const void* const* grads, const uint64_t* n_elems,
                                 uint32_t count, edgc_dtype dtype, uint64_t stride, uint32_t chunk,
                                           uint64_t seed, uint64_t step, uint32_t bins, const float* range,
                                           edgc_entropy_result* out, uint64_t* counts_out, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!grads || !n_elems || !out) return fail(ctx, EDGC_EINVAL, "null grads, n_elems or out");
    if (count == 0 || count > static_cast<uint32_t>(kMaxEntGroup))
        return fail(ctx, EDGC_EINVAL, "an entropy estimate takes 1 to 32 buffers");
    if (dtype != EDGC_F32 && dtype != EDGC_BF16) return fail(ctx, EDGC_EINVAL, "unknown dtype");
    if (int rc = check_sampler_args(ctx, stride, chunk)) return rc;
    if (static_scratch) {
        if (bins == 0 || bins > kStaticMaxBins)
            return fail(ctx, EDGC_EINVAL, "edgc_entropy_estimate_noalloc takes 1 to 65536 bins");
    } else if (bins == 0 || bins > ctx->max_bins) {
        return fail(ctx, EDGC_EINVAL, "bins == 0 or bins > max_bins");
    }
    if (range && !(range[0] <= range[1])) return fail(ctx, EDGC_EINVAL, "range needs lo <= hi");
    if (counts_out && !aligned_to(counts_out, 8)) return fail(ctx, EDGC_EINVAL, "counts misaligned");
    for (uint32_t i = 0; i < count; ++i) {
        if (!grads[i]) return fail(ctx, EDGC_EINVAL, "null grad");
        if (!aligned_to(grads[i], dtype == EDGC_F32 ? 4 : 2)) return fail(ctx, EDGC_EINVAL, "grad misaligned");
        if (n_elems[i] > (1ull << 44)) return fail(ctx, EDGC_EINVAL, "n_elems too large");
    }
    EntGroup g{};
    g.count = count;
    // one vector width for the whole group: scalar loads as soon as one buffer needs them
    for (int pass = 0; pass < 2; ++pass) {
        bool uniform = true;
        g.n_items = g.n_sampled = 0;
        for (uint32_t i = 0; i < count; ++i) {
            g.base[i] = grads[i];
            g.geom[i] = make_geom(grads[i], dtype, n_elems[i], stride, chunk, seed, step, pass == 0);
            g.n_items += g.geom[i].n_items;
            g.n_sampled += g.geom[i].n_sampled;
            uniform = uniform && (g.geom[i].vec > 1) == (g.geom[0].vec > 1);
        }
        if (uniform) break;
    }
    if (g.n_sampled == 0) return fail(ctx, EDGC_ENONFINITE, "the sampling predicate selects no element");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    if (static_scratch)
        return launch_entropy_static(ctx, g, dtype, bins, range, out, counts_out, static_cast<hipStream_t>(hip_stream));
    return launch_entropy(ctx, g, dtype, bins, range, out, counts_out, static_cast<hipStream_t>(hip_stream));
}

extern "C" int edgc_entropy_estimate_batch(edgc_ctx* ctx, const void* const* grads, const uint64_t* n_elems,
                                           uint32_t count, edgc_dtype dtype, uint64_t stride, uint32_t chunk,
                                           uint64_t seed, uint64_t step, uint32_t bins, const float* range,
                                           edgc_entropy_result* out, uint64_t* counts_out, void* hip_stream)
{
    return entropy_estimate_impl(ctx, false, grads, n_elems, count, dtype, stride, chunk, seed, step, bins, range,
                                 out, counts_out, hip_stream);
}

extern "C" int edgc_entropy_estimate_noalloc(edgc_ctx* ctx, const void* grad, edgc_dtype dtype,
                                             uint64_t n_elems, uint64_t stride, uint32_t chunk, uint64_t seed,
                                             uint64_t step, uint32_t bins, const float* range,
                                             edgc_entropy_result* out, uint64_t* counts_out, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!grad || !out) return fail(ctx, EDGC_EINVAL, "null grad or out");
    return entropy_estimate_impl(ctx, true, &grad, &n_elems, 1, dtype, stride, chunk, seed, step, bins, range, out,
                                 counts_out, hip_stream);
}


extern "C" int edgc_sample_indices(edgc_ctx* ctx, uint64_t n_elems, uint64_t stride, uint32_t chunk,
                                   uint64_t seed, uint64_t step, uint64_t* idx_out, uint64_t cap,
                                   uint64_t* n_out, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!n_out) return fail(ctx, EDGC_EINVAL, "null n_out");
    if (int rc = check_sampler_args(ctx, stride, chunk)) return rc;
    // layout of the indices does not depend on dtype or alignment: use the scalar geometry
    SampleGeom g = make_geom(reinterpret_cast<const void*>(uintptr_t{1}), EDGC_F32, n_elems, stride,
                             chunk, seed, step);
    *n_out = g.n_sampled;
    if (!idx_out || cap == 0) return EDGC_OK;
    if (!aligned_to(idx_out, 8)) return fail(ctx, EDGC_EINVAL, "idx_out misaligned");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    return launch_sample_indices(ctx, g, idx_out, cap, static_cast<hipStream_t>(hip_stream));
}

extern "C" int edgc_init_q(edgc_ctx* ctx, float* Q, uint32_t n, uint32_t ldq, uint32_t col_begin,
                           uint32_t col_end, uint64_t seed, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!Q || col_begin > col_end || col_end > ldq) return fail(ctx, EDGC_EINVAL, "bad Q columns");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    return launch_init_q(ctx, Q, n, ldq, col_begin, col_end, seed, static_cast<hipStream_t>(hip_stream));
}

static int check_factor_args(edgc_ctx* ctx, const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                             uint32_t m, uint32_t n, uint32_t r, uint64_t ld, uint64_t max_rows,
                             uint64_t max_cols)
{
    if (!P || !Q) return fail(ctx, EDGC_EINVAL, "null P or Q");
    if (m == 0 || n == 0) return fail(ctx, EDGC_EINVAL, "empty matrix");
    if (m > max_rows || n > max_cols) return fail(ctx, EDGC_EINVAL, "matrix larger than the context");
    if (r == 0 || r > m || r > n || r > ctx->max_rank) return fail(ctx, EDGC_EINVAL, "rank out of range");
    if (ld < n || ldp < r || ldq < r) return fail(ctx, EDGC_EINVAL, "leading dimension too small");
    if (m > kMaxDim || n > kMaxDim || ld > kMaxDim)
        return fail(ctx, EDGC_EINVAL, "rows, columns and leading dimensions are limited to 2^28");
    if (ldp % 4 || ldq % 4 || !aligned_to(P, 16) || !aligned_to(Q, 16))
        return fail(ctx, EDGC_EINVAL, "P and Q need 16-byte alignment and leading dimensions that are multiples of 4");
    return EDGC_OK;
}

// scratch of the context itself: serves one tensor
static void own_scratch(edgc_ctx* ctx, TensorArgs& t, TensorScratch& cap)
{
    Scratch& s = ctx->s;
    t.part = s.part; t.gram_part = s.gram_part; t.gram = s.gram; t.rinv = s.rinv; t.pt = s.pt;
    cap.part_elems = s.part_elems;
    cap.gram_part_elems = s.gram_part_elems;
}

namespace {

// The single-tensor calls with the deferred flag of the batched ones (a group of one on the
// context's own scratch); the public single-tensor entry points pass 0.
int compress_one(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint32_t m, uint32_t n,
                 uint64_t ld, float* residual, int residual_is_zero, float* Q, uint32_t ldq,
                 float* P, uint32_t ldp, uint32_t r, uint32_t power_iters, uint32_t defer, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!grad || !residual) return fail(ctx, EDGC_EINVAL, "null grad or residual");
    if (dtype != EDGC_F32 && dtype != EDGC_BF16) return fail(ctx, EDGC_EINVAL, "unknown dtype");
    if (int rc = check_factor_args(ctx, P, ldp, Q, ldq, m, n, r, ld, ctx->max_rows, ctx->max_cols)) return rc;
    if (power_iters == 0) return fail(ctx, EDGC_EINVAL, "power_iters must be >= 1");
    if (!aligned_to(grad, dtype == EDGC_F32 ? 4 : 2) || !aligned_to(residual, 4))
        return fail(ctx, EDGC_EINVAL, "grad or residual misaligned");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    Group g{};
    g.count = 1;
    g.r = r;
    g.defer = defer;
    TensorArgs& t = g.t[0];
    t.G = grad; t.ldg = ld; t.E = residual; t.e_zero = residual_is_zero ? 1 : 0;
    t.Q = Q; t.ldq = ldq; t.P = P; t.ldp = ldp; t.m = m; t.n = n;
    TensorScratch cap;
    own_scratch(ctx, t, cap);
    return launch_compress(ctx, g, &cap, dtype, power_iters, static_cast<hipStream_t>(hip_stream));
}

int decompress_one(edgc_ctx* ctx, const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                   uint32_t m, uint32_t n, uint32_t r, float* residual, void* grad_out,
                   edgc_dtype dtype, uint64_t ld, uint32_t defer, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (!residual || !grad_out) return fail(ctx, EDGC_EINVAL, "null residual or grad_out");
    if (dtype != EDGC_F32 && dtype != EDGC_BF16) return fail(ctx, EDGC_EINVAL, "unknown dtype");
    if (int rc = check_factor_args(ctx, P, ldp, Q, ldq, m, n, r, ld, ctx->max_rows, ctx->max_cols)) return rc;
    if (!aligned_to(grad_out, dtype == EDGC_F32 ? 4 : 2) || !aligned_to(residual, 4))
        return fail(ctx, EDGC_EINVAL, "grad_out or residual misaligned");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    Group g{};
    g.count = 1;
    g.r = r;
    g.defer = defer;
    TensorArgs& t = g.t[0];
    t.E = residual; t.Q = const_cast<float*>(Q); t.ldq = ldq; t.P = const_cast<float*>(P); t.ldp = ldp;
    t.out = grad_out; t.ldo = ld; t.m = m; t.n = n;
    return launch_decompress(ctx, g, dtype, static_cast<hipStream_t>(hip_stream));
}

}  // namespace

extern "C" int edgc_compress(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint32_t m, uint32_t n,
                             uint64_t ld, float* residual, int residual_is_zero, float* Q, uint32_t ldq,
                             float* P, uint32_t ldp, uint32_t r, uint32_t power_iters, void* hip_stream)
{
    return compress_one(ctx, grad, dtype, m, n, ld, residual, residual_is_zero, Q, ldq, P, ldp, r, power_iters, 0,
                        hip_stream);
}

extern "C" int edgc_decompress(edgc_ctx* ctx, const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                               uint32_t m, uint32_t n, uint32_t r, float* residual, void* grad_out,
                               edgc_dtype dtype, uint64_t ld, void* hip_stream)
{
    return decompress_one(ctx, P, ldp, Q, ldq, m, n, r, residual, grad_out, dtype, ld, 0, hip_stream);
}

// ---------------------------------------------------------------------------
// Batched calls: all 2-D gradients of a pipeline stage in one launch sequence.
// ---------------------------------------------------------------------------
extern "C" int edgc_tensor_bypassed(uint32_t m, uint32_t n, uint32_t r)
{
    if (m == 0 || n == 0 || r == 0) return EDGC_EINVAL;
    if (m == 1 || n == 1) return 1;
    return (static_cast<uint64_t>(m) + n) * r >= static_cast<uint64_t>(m) * n ? 1 : 0;
}

extern "C" int edgc_reserve_batch(edgc_ctx* ctx, const uint32_t* rows, const uint32_t* cols, uint32_t count)
{
    if (!ctx) return EDGC_EINVAL;
    if (count && (!rows || !cols)) return fail(ctx, EDGC_EINVAL, "null shape arrays");
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    EDGC_HIP_TRY(ctx, hipDeviceSynchronize());          // nothing may still be using the old slots
    free_batch(ctx);
    const uint64_t rp = (ctx->max_rank <= 32) ? 32 : (ctx->max_rank <= 64 ? 64 : 128);
    ctx->batch.resize(count);
    bool ok = true;
    for (uint32_t i = 0; i < count && ok; ++i) {
        BatchSlot& b = ctx->batch[i];
        b.rows = rows[i];
        b.cols = cols[i];
        if (rows[i] == 0 || cols[i] == 0 || rows[i] == 1 || cols[i] == 1) continue;   // never compressed
        if (rows[i] > kMaxDim || cols[i] > kMaxDim) {
            free_batch(ctx);
            return fail(ctx, EDGC_EINVAL, "rows and columns of a compressed tensor are limited to 2^28");
        }
        const uint64_t rows_pad = (static_cast<uint64_t>(rows[i]) + 63) / 64 * 64;
        b.cap.part_elems = compress_part_elems(rows[i], cols[i], ctx->max_rank, ctx->num_cu);
        b.cap.gram_part_elems = (rows_pad / 64) * 36ull * 256ull;
        ok = ok && dev_alloc(&b.part, b.cap.part_elems) == hipSuccess;
        ok = ok && dev_alloc(&b.gram_part, b.cap.gram_part_elems) == hipSuccess;
        ok = ok && dev_alloc(&b.gram, static_cast<size_t>(36) * 256) == hipSuccess;
        ok = ok && dev_alloc(&b.rinv, rinv_elems(ctx->max_rank)) == hipSuccess;
        ok = ok && hipMalloc(&b.pt, 2ull * rp * rows_pad * 2ull) == hipSuccess;
    }
    if (!ok) {
        (void)hipGetLastError();
        free_batch(ctx);
        return fail(ctx, EDGC_ENOMEM, "batch scratch allocation failed");
    }
    return EDGC_OK;
}

namespace {

// Checks one descriptor; returns 1 when the tensor is sent as it stands, 0 when it is
// compressed, < 0 on error.
int check_batch_tensor(edgc_ctx* ctx, const edgc_tensor& d, uint32_t i, edgc_dtype dtype, uint32_t r,
                       bool need_grad, bool need_out)
{
    if (d.m == 0 || d.n == 0) return fail(ctx, EDGC_EINVAL, "empty tensor in batch");
    if ((need_grad && !d.grad) || (need_out && !d.grad_out)) return fail(ctx, EDGC_EINVAL, "null gradient pointer in batch");
    const uint32_t esz = dtype == EDGC_F32 ? 4 : 2;
    if ((need_grad && (!aligned_to(d.grad, esz) || d.ld < d.n)) ||
        (need_out && (!aligned_to(d.grad_out, esz) || d.ld_out < d.n)))
        return fail(ctx, EDGC_EINVAL, "gradient misaligned or leading dimension too small in batch");
    if (edgc_tensor_bypassed(d.m, d.n, r) == 1) return 1;
    const BatchSlot& b = ctx->batch[i];
    if (d.m > b.rows || d.n > b.cols || !b.part)
        return fail(ctx, EDGC_EINVAL, "tensor larger than the batch slot reserved for its position");
    if (!d.residual || !aligned_to(d.residual, 4)) return fail(ctx, EDGC_EINVAL, "null or misaligned residual in batch");
    if (int rc = check_factor_args(ctx, d.P, d.ldp, d.Q, d.ldq, d.m, d.n, r, d.n, b.rows, b.cols)) return rc;
    if ((need_grad && d.ld > kMaxDim) || (need_out && d.ld_out > kMaxDim))
        return fail(ctx, EDGC_EINVAL, "rows, columns and leading dimensions are limited to 2^28");
    return 0;
}

// The deferred flag of a call: every compressed tensor must carry the same one.
// Returns 0 / 1, or < 0 when the descriptors disagree or the flag is neither.
int batch_deferred(edgc_ctx* ctx, const edgc_tensor* tensors, const std::vector<int>& kind)
{
    int flag = -1;
    for (size_t i = 0; i < kind.size(); ++i) {
        if (kind[i] == 1) continue;
        if (tensors[i].deferred > 1) return fail(ctx, EDGC_EINVAL, "edgc_tensor.deferred must be 0 or 1");
        const int f = static_cast<int>(tensors[i].deferred);
        if (flag >= 0 && f != flag)
            return fail(ctx, EDGC_EINVAL, "the tensors of one batch call must agree in `deferred`");
        flag = f;
    }
    return flag < 0 ? 0 : flag;
}

}  // namespace

namespace {

// phase: 0 the whole compress, 1 up to P = D Q, 2 from P as it stands (launch_compress)
int compress_batch_impl(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count, edgc_dtype dtype,
                        uint32_t r, uint32_t power_iters, int phase, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (count == 0) return EDGC_OK;
    if (!tensors) return fail(ctx, EDGC_EINVAL, "null tensor list");
    if (dtype != EDGC_F32 && dtype != EDGC_BF16) return fail(ctx, EDGC_EINVAL, "unknown dtype");
    if (r == 0 || r > ctx->max_rank) return fail(ctx, EDGC_EINVAL, "rank out of range");
    if (power_iters == 0) return fail(ctx, EDGC_EINVAL, "power_iters must be >= 1");
    if (count > ctx->batch.size()) return fail(ctx, EDGC_EINVAL, "more tensors than reserved batch slots");
    std::vector<int> kind(count);
    for (uint32_t i = 0; i < count; ++i) {
        kind[i] = check_batch_tensor(ctx, tensors[i], i, dtype, r, phase != 2, false);
        if (kind[i] < 0) return kind[i];
    }
    const int defer = phase == 2 ? 0 : batch_deferred(ctx, tensors, kind);   // the second phase reads D as it stands
    if (defer < 0) return defer;
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Group g{};
    TensorScratch cap[kMaxGroup];
    g.r = r;
    g.defer = static_cast<uint32_t>(defer);
    auto flush = [&]() -> int {
        if (g.count == 0) return EDGC_OK;
        const int rc = launch_compress(ctx, g, cap, dtype, power_iters, st, phase);
        g = Group{};
        g.r = r;
        g.defer = static_cast<uint32_t>(defer);
        return rc;
    };
    for (uint32_t i = 0; i < count; ++i) {
        if (kind[i] == 1) continue;
        const edgc_tensor& d = tensors[i];
        const BatchSlot& b = ctx->batch[i];
        TensorArgs& t = g.t[g.count];
        t.G = d.grad; t.ldg = d.ld; t.E = d.residual; t.e_zero = d.residual_is_zero ? 1 : 0;
        t.Q = d.Q; t.ldq = d.ldq; t.P = d.P; t.ldp = d.ldp; t.m = d.m; t.n = d.n;
        t.part = b.part; t.gram_part = b.gram_part; t.gram = b.gram; t.rinv = b.rinv; t.pt = b.pt;
        cap[g.count] = b.cap;
        if (++g.count == kMaxGroup)
            if (int rc = flush()) return rc;
    }
    return flush();
}

}  // namespace

extern "C" int edgc_compress_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                                   edgc_dtype dtype, uint32_t r, uint32_t power_iters, void* hip_stream)
{
    return compress_batch_impl(ctx, tensors, count, dtype, r, power_iters, 0, hip_stream);
}

extern "C" int edgc_compress_p_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                                     edgc_dtype dtype, uint32_t r, void* hip_stream)
{
    return compress_batch_impl(ctx, tensors, count, dtype, r, 1, 1, hip_stream);
}

extern "C" int edgc_compress_q_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                                     edgc_dtype dtype, uint32_t r, void* hip_stream)
{
    return compress_batch_impl(ctx, tensors, count, dtype, r, 1, 2, hip_stream);
}

namespace {

// Shared by edgc_decompress_batch and edgc_residual_materialize_batch (with_out = false: the
// reconstruction is not written, E = D - M^ alone).
int decompress_batch_impl(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count, edgc_dtype dtype,
                          uint32_t r, bool with_out, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (count == 0) return EDGC_OK;
    if (!tensors) return fail(ctx, EDGC_EINVAL, "null tensor list");
    if (dtype != EDGC_F32 && dtype != EDGC_BF16) return fail(ctx, EDGC_EINVAL, "unknown dtype");
    if (r == 0 || r > ctx->max_rank) return fail(ctx, EDGC_EINVAL, "rank out of range");
    if (count > ctx->batch.size()) return fail(ctx, EDGC_EINVAL, "more tensors than reserved batch slots");
    std::vector<int> kind(count);
    for (uint32_t i = 0; i < count; ++i) {
        kind[i] = check_batch_tensor(ctx, tensors[i], i, dtype, r, false, with_out);
        if (kind[i] < 0) return kind[i];
        if (with_out && kind[i] == 1 && !tensors[i].grad) return fail(ctx, EDGC_EINVAL, "null gradient pointer in batch");
    }
    int defer = 0;
    if (with_out) {
        defer = batch_deferred(ctx, tensors, kind);
        if (defer < 0) return defer;
    }
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Group g{};
    g.r = r;
    g.defer = static_cast<uint32_t>(defer);
    auto flush = [&]() -> int {
        if (g.count == 0) return EDGC_OK;
        const int rc = launch_decompress(ctx, g, dtype, st);
        g = Group{};
        g.r = r;
        g.defer = static_cast<uint32_t>(defer);
        return rc;
    };
    const uint32_t esz = dtype == EDGC_F32 ? 4 : 2;
    for (uint32_t i = 0; i < count; ++i) {
        const edgc_tensor& d = tensors[i];
        if (kind[i] == 1) {                      // sent as it stands: hand the gradient on
            if (with_out)
                if (int rc = launch_copy_rows(ctx, d.grad, d.ld, d.grad_out, d.ld_out, d.m, d.n, esz, st)) return rc;
            continue;
        }
        TensorArgs& t = g.t[g.count];
        t.E = d.residual; t.Q = d.Q; t.ldq = d.ldq; t.P = d.P; t.ldp = d.ldp;
        t.out = with_out ? d.grad_out : nullptr; t.ldo = with_out ? d.ld_out : 0; t.m = d.m; t.n = d.n;
        if (++g.count == kMaxGroup)
            if (int rc = flush()) return rc;
    }
    return flush();
}

}  // namespace

extern "C" int edgc_decompress_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                                     edgc_dtype dtype, uint32_t r, void* hip_stream)
{
    return decompress_batch_impl(ctx, tensors, count, dtype, r, true, hip_stream);
}

extern "C" int edgc_residual_materialize_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                                               edgc_dtype dtype, uint32_t r, void* hip_stream)
{
    return decompress_batch_impl(ctx, tensors, count, dtype, r, false, hip_stream);
}

// Sec. IV-D-1 asks for T_compress and T_decompress measured on the system at hand: time this
// library's own two calls at every candidate rank.
extern "C" int edgc_measure_rank_costs(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint32_t m,
                                       uint32_t n, uint64_t ld, float* residual, float* Q, uint32_t ldq,
                                       float* P, uint32_t ldp, void* grad_out, const uint32_t* ranks,
                                       uint32_t n_ranks, uint32_t reps, int deferred,
                                       edgc_rank_cost* costs_out, void* hip_stream)
{
    if (!ctx) return EDGC_EINVAL;
    if (deferred != 0 && deferred != 1) return fail(ctx, EDGC_EINVAL, "deferred must be 0 or 1");
    const uint32_t defer = static_cast<uint32_t>(deferred);
    if (!ranks || !costs_out || n_ranks == 0 || reps == 0)
        return fail(ctx, EDGC_EINVAL, "null ranks/costs_out, n_ranks == 0 or reps == 0");
    if (grad_out == grad) return fail(ctx, EDGC_EINVAL, "grad_out must not alias grad while measuring");
    for (uint32_t i = 0; i < n_ranks; ++i)
        if (ranks[i] == 0 || (i && ranks[i] <= ranks[i - 1])) return fail(ctx, EDGC_EINVAL, "ranks must ascend");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    int rc = EDGC_OK;
    auto hip_ok = [&](hipError_t e, const char* what) {
        if (e == hipSuccess) return true;
        rc = fail(ctx, EDGC_EHIP, what);
        return false;
    };
    for (auto& e : ev)
        if (!hip_ok(hipEventCreate(&e), "hipEventCreate")) break;
    for (uint32_t i = 0; rc == EDGC_OK && i < n_ranks; ++i) {
        const uint32_t r = ranks[i];
        double t_c = 0.0, t_d = 0.0;
        // repetition 0 is untimed and starts from a zero residual and fresh Q columns
        rc = edgc_init_q(ctx, Q, n, ldq, 0, r, 0x5eedULL + r, hip_stream);
        for (uint32_t rep = 0; rc == EDGC_OK && rep <= reps; ++rep) {
            if (!hip_ok(hipEventRecord(ev[0], st), "hipEventRecord")) break;
            // a deferred compress needs D and the factors of a step before it: not in repetition 0
            rc = compress_one(ctx, grad, dtype, m, n, ld, residual, rep == 0, Q, ldq, P, ldp, r, 1,
                              rep == 0 ? 0u : defer, hip_stream);
            if (rc != EDGC_OK) break;
            if (!hip_ok(hipEventRecord(ev[1], st), "hipEventRecord")) break;
            rc = decompress_one(ctx, P, ldp, Q, ldq, m, n, r, residual, grad_out, dtype, ld, defer, hip_stream);
            if (rc != EDGC_OK) break;
            if (!hip_ok(hipEventRecord(ev[2], st), "hipEventRecord")) break;
            if (!hip_ok(hipEventSynchronize(ev[2]), "hipEventSynchronize")) break;
            if (rep == 0) continue;
            float ms_c = 0.f, ms_d = 0.f;
            if (!hip_ok(hipEventElapsedTime(&ms_c, ev[0], ev[1]), "hipEventElapsedTime")) break;
            if (!hip_ok(hipEventElapsedTime(&ms_d, ev[1], ev[2]), "hipEventElapsedTime")) break;
            t_c += ms_c;
            t_d += ms_d;
        }
        costs_out[i].rank = r;
        costs_out[i]._pad = 0;
        costs_out[i].t_compress = 1e-3 * t_c / reps;
        costs_out[i].t_decompress = 1e-3 * t_d / reps;
        costs_out[i].bytes_compressed = 4.0 * (static_cast<double>(m) + static_cast<double>(n)) * r;
    }
    for (auto& e : ev)
        if (e) (void)hipEventDestroy(e);
    return rc;
}
