// Down-sampled gradient entropy on gfx950 (GDS, Sec. IV-B; Definition 1 / Eq. (1)
// estimated with an equal-width histogram).
//
// Two streaming kernels over the sampled chunks plus nothing else:
//   k_minmax  range of the finite sample: per-lane min/max, wavefront DPP
//             reduction, LDS across the block's waves, last-block finish
//   k_hist    bin index in fp32 (separately rounded subtract / multiply, the
//             scale comes from one correctly rounded division), LDS histogram
//             with lane-interleaved replicas so equal bins in one wavefront hit
//             different banks, flush to 64-bit global counters, and the last
//             block reduces the counters to the Shannon entropy in fp64
// The chunk-strided sample is read with 16-byte loads whenever chunks are a
// multiple of the vector width, so a wavefront touches whole cache lines.
// Both kernels take a list of buffers (EntGroup): the estimate is over the union
// of the buffers' samples (one entropy for a pipeline stage whose gradients are
// separate tensors); a single buffer is a list of one.  The result goes straight
// into the caller's pinned host memory when it is device-accessible.
#include "edgc_internal.h"

#include <math.h>

namespace edgc {

struct RangeParams {
    float lo, hi, w, scale;
};

constexpr int kMMBlock   = 256;
constexpr int kMMBlockFat = 1024;                 // large samples: one block per CU
constexpr uint64_t kBigSampleItems = 8ull << 20;  // items (16 bytes each) from which a sample counts as large
constexpr int kHistBlock = 512;
constexpr int kSmallSampleBlocks = 16;   // blocks the kernels of a sample of up to 512 Ki items get at most
constexpr int kHistBlockFat = 1024;   // when the LDS histogram leaves room for one block per CU

// ---------------------------------------------------------------------------
// wavefront reductions with DPP row shifts / row broadcasts (64 lanes)
// ---------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float identity, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v),
                                                      CTRL, ROW_MASK, 0xf, false));
}

// Result is valid in lane 63 and returned to every lane through a read-lane.
template <bool IS_MIN>
__device__ __forceinline__ float wave_reduce_minmax(float v)
{
    const float id = IS_MIN ? INFINITY : -INFINITY;
#define EDGC_OP(a, b) (IS_MIN ? fminf((a), (b)) : fmaxf((a), (b)))
    v = EDGC_OP(v, (dpp_move<0x111, 0xf>(id, v)));   // row_shr:1
    v = EDGC_OP(v, (dpp_move<0x112, 0xf>(id, v)));   // row_shr:2
    v = EDGC_OP(v, (dpp_move<0x114, 0xf>(id, v)));   // row_shr:4
    v = EDGC_OP(v, (dpp_move<0x118, 0xf>(id, v)));   // row_shr:8  -> lane 15 of each row
    v = EDGC_OP(v, (dpp_move<0x142, 0xa>(id, v)));   // row_bcast:15 into rows 1 and 3
    v = EDGC_OP(v, (dpp_move<0x143, 0xc>(id, v)));   // row_bcast:31 into rows 2 and 3
#undef EDGC_OP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;   // lane 0
}

// ---------------------------------------------------------------------------
// sample addressing
// ---------------------------------------------------------------------------
template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
    static __device__ __forceinline__ float widen(float x) { return x; }
};
template <> struct ElemTraits<uint16_t> {   // raw bf16 bits
    static __device__ __forceinline__ float widen(uint16_t h)
    {
        return __uint_as_float(static_cast<uint32_t>(h) << 16);
    }
};

// Loads the VEC elements of one item starting at element i0; elements at or
// beyond n are reported invalid.  Full items use one 16-byte load.
template <typename T, int VEC>
__device__ __forceinline__ uint32_t load_item(const T* __restrict__ g, uint64_t i0, uint64_t n,
                                              float (&v)[VEC])
{
    if constexpr (VEC == 1) {
        v[0] = ElemTraits<T>::widen(g[i0]);
        return 1u;
    } else {
        if (i0 + VEC <= n) {
            if constexpr (sizeof(T) == 4) {
                const float4 q = *reinterpret_cast<const float4*>(g + i0);
                v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
            } else {
                const uint4 q = *reinterpret_cast<const uint4*>(g + i0);
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    v[2 * p]     = __uint_as_float(w[p] << 16);
                    v[2 * p + 1] = __uint_as_float(w[p] & 0xffff0000u);
                }
            }
            return (1u << VEC) - 1u;
        }
        uint32_t mask = 0;
#pragma unroll
        for (int p = 0; p < VEC; ++p) {
            v[p] = 0.0f;
            if (i0 + p < n) { v[p] = ElemTraits<T>::widen(g[i0 + p]); mask |= 1u << p; }
        }
        return mask;
    }
}

// The VEC elements of a whole item from its 16 raw bytes.
template <typename T, int VEC>
__device__ __forceinline__ void unpack_item(const uint4& q, float (&v)[VEC])
{
    static_assert(VEC * sizeof(T) == 16, "a vector item is 16 bytes");
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int p = 0; p < 4; ++p) v[p] = __uint_as_float(w[p]);
    } else {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            v[2 * p]     = __uint_as_float(w[p] << 16);
            v[2 * p + 1] = __uint_as_float(w[p] & 0xffff0000u);
        }
    }
}

// Walks the items owned by one thread: item t, t + G, t + 2G, ... without a
// division in the loop.  item -> (k-th sampled chunk, e-th item in it).
struct ItemCursor {
    uint64_t item, k;
    uint32_t e;
    uint64_t dk;
    uint32_t de;
    __device__ __forceinline__ void init(uint64_t first, uint64_t step, uint32_t ipc)
    {
        item = first;
        k = first / ipc;
        e = static_cast<uint32_t>(first - k * ipc);
        dk = step / ipc;
        de = static_cast<uint32_t>(step - dk * ipc);
    }
    __device__ __forceinline__ void advance(uint64_t step, uint32_t ipc)
    {
        item += step;
        k += dk;
        e += de;
        if (e >= ipc) { e -= ipc; ++k; }
    }
    __device__ __forceinline__ uint64_t elem0(const SampleGeom& g, int vec) const
    {
        return (g.slot + k * g.stride) * g.chunk + static_cast<uint64_t>(e) * vec;
    }
};

__device__ __forceinline__ bool finite_f32(float x)
{
    return (__float_as_uint(x) & 0x7f800000u) != 0x7f800000u;
}

// The estimate from sum c log2 c (`acc`) and sum c (`tot`) over the bins, by one thread:
// H = log2 n - (1/n) sum c log2 c in fp64, and the result record.
__device__ __forceinline__ void emit_result(double acc, double tot, uint32_t bins, const RangeParams* rp,
                                            unsigned long long n_sampled, edgc_entropy_result* res)
{
    edgc_entropy_result r;
    r.lo = rp->lo; r.hi = rp->hi;
    r.n_sampled = n_sampled;
    // every finite element of the sample was counted in exactly one bin (values outside a caller's
    // range in the edge bins), so what the bins do not hold is the non-finite part; the counts are
    // integers below 2^53, their sum in fp64 is exact
    r.n_nonfinite = n_sampled - static_cast<unsigned long long>(tot);
    r._pad = 0;
    if (tot > 0.0) {
        double H = log2(tot) - acc / tot;
        if (H < 0.0) H = 0.0;
        const double w = static_cast<double>(rp->w);
        r.H_bits = H;
        r.h_diff_nats = (w > 0.0) ? H * 0.69314718055994530942 + log(w / static_cast<double>(bins))
                                  : -INFINITY;
        r.status = EDGC_OK;
    } else {
        r.H_bits = NAN; r.h_diff_nats = NAN;
        r.status = EDGC_ENONFINITE;
    }
    *res = r;
    __threadfence_system();       // `res` may be the caller's pinned host memory
}

__device__ __forceinline__ void entropy_term(unsigned long long c, double& acc, double& tot)
{
    if (c) {
        const double d = static_cast<double>(c);
        acc += d * log2(d);
        tot += d;
    }
}

// Sums the threads' (acc, tot) over the block; thread 0 returns the totals.
template <int BLOCK>
__device__ __forceinline__ void block_sum_pair(double& acc, double& tot)
{
    __shared__ double s_a[BLOCK / 64], s_b[BLOCK / 64];
    acc = wave_sum_f64(acc);
    tot = wave_sum_f64(tot);
    __syncthreads();              // the arrays may still be read from an earlier call
    if ((threadIdx.x & 63) == 0) { s_a[threadIdx.x >> 6] = acc; s_b[threadIdx.x >> 6] = tot; }
    __syncthreads();
    if (threadIdx.x == 0) {
        acc = 0.0; tot = 0.0;
        for (int w = 0; w < BLOCK / 64; ++w) { acc += s_a[w]; tot += s_b[w]; }
    }
}

// Shannon entropy of the 64-bit counters and the result record, by one whole block (the last one of a
// grid).
template <int BLOCK>
__device__ __forceinline__ void finish_entropy(const unsigned long long* counts, uint32_t bins,
                                               const RangeParams* rp, unsigned long long n_sampled,
                                               edgc_entropy_result* res)
{
    double acc = 0.0, tot = 0.0;
    for (uint32_t i = threadIdx.x; i < bins; i += BLOCK)
        entropy_term(__hip_atomic_load(&counts[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), acc, tot);
    block_sum_pair<BLOCK>(acc, tot);
    if (threadIdx.x == 0) emit_result(acc, tot, bins, rp, n_sampled, res);
}

// ---------------------------------------------------------------------------
// kernel 1: range of the finite sample
// ---------------------------------------------------------------------------
template <typename T, int VEC, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_minmax(const EntGroup grp,
                                                     float* __restrict__ part,
                                                     unsigned int* done, RangeParams* rp,
                                                     float fbins, unsigned long long* counts,
                                                     uint32_t bins, const unsigned int* gate)
{
    // behind the one-pass kernel of bf16 samples: only when that one reported a counter overflow
    if (gate && __hip_atomic_load(gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    const uint64_t G = static_cast<uint64_t>(gridDim.x) * BLOCK;
    const uint64_t gtid = static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x;
    // the histogram kernel that follows on the stream accumulates into zeroed counters
    for (uint64_t b = gtid; b < bins; b += G) counts[b] = 0ull;

    float lo = INFINITY, hi = -INFINITY;
    constexpr int U = 4;
    for (uint32_t ti = 0; ti < grp.count; ++ti) {
    const SampleGeom& geom = grp.geom[ti];
    const T* __restrict__ g = static_cast<const T*>(grp.base[ti]);
    // a block takes one contiguous range of the buffer's items (the sets are the same as with any
    // other assignment; consecutive rounds of a block then read consecutive memory)
    const uint64_t per = (geom.n_items + gridDim.x - 1) / gridDim.x;
    const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * per;
    const uint64_t end = min(begin + per, geom.n_items);
    ItemCursor cur;
    cur.init(begin + threadIdx.x, BLOCK, geom.ipc);
    if constexpr (VEC > 1) {
        // rounds of U whole items per thread with the next round's loads in flight (see k_hist)
        const uint64_t fast_end = (geom.n_items >= geom.ipc) ? min(end, geom.n_items - geom.ipc) : 0;
        auto round_fits = [&]() { return cur.item + static_cast<uint64_t>(U - 1) * BLOCK < fast_end; };
        auto fetch_raw = [&](uint4 (&raw)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                raw[u] = *reinterpret_cast<const uint4*>(g + cur.elem0(geom, VEC));
                cur.advance(BLOCK, geom.ipc);
            }
        };
        auto fold_raw = [&](const uint4 (&raw)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float v[VEC];
                unpack_item<T, VEC>(raw[u], v);
#pragma unroll
                for (int p = 0; p < VEC; ++p) {
                    const bool fin = finite_f32(v[p]);
                    lo = fminf(lo, fin ? v[p] : lo);
                    hi = fmaxf(hi, fin ? v[p] : hi);
                }
            }
        };
        if (round_fits()) {
            uint4 ra[U], rb[U];
            fetch_raw(ra);
            while (true) {
                if (!round_fits()) { fold_raw(ra); break; }
                fetch_raw(rb);
                fold_raw(ra);
                if (!round_fits()) { fold_raw(rb); break; }
                fetch_raw(ra);
                fold_raw(rb);
            }
        }
    }
    while (cur.item < end) {
        float v[U][VEC];
        uint32_t mask[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mask[u] = 0;
            if (cur.item < end) {
                const uint64_t i0 = cur.elem0(geom, VEC);
                if (i0 < geom.n) mask[u] = load_item<T, VEC>(g, i0, geom.n, v[u]);
            }
            cur.advance(BLOCK, geom.ipc);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (mask[u] == (1u << VEC) - 1u) {
                // a whole item: no branch per element, a non-finite value stands in as the bound itself
#pragma unroll
                for (int p = 0; p < VEC; ++p) {
                    const float x = v[u][p];
                    const bool fin = finite_f32(x);
                    lo = fminf(lo, fin ? x : lo);
                    hi = fmaxf(hi, fin ? x : hi);
                }
            } else {
#pragma unroll
                for (int p = 0; p < VEC; ++p)
                    if (((mask[u] >> p) & 1u) && finite_f32(v[u][p])) {
                        lo = fminf(lo, v[u][p]);
                        hi = fmaxf(hi, v[u][p]);
                    }
            }
        }
    }
    }

    __shared__ float s_lo[BLOCK / 64], s_hi[BLOCK / 64];
    __shared__ bool s_last;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    lo = wave_reduce_minmax<true>(lo);
    hi = wave_reduce_minmax<false>(hi);
    if (lane == 0) { s_lo[wave] = lo; s_hi[wave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < BLOCK / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
        part[2 * blockIdx.x]     = lo;
        part[2 * blockIdx.x + 1] = hi;
        __threadfence();
        const unsigned int ticket = atomicAdd(done, 1u);
        s_last = (ticket == gridDim.x - 1);
    }
    __syncthreads();
    if (!s_last) return;

    // last block: fold the per-block partials
    __threadfence();
    lo = INFINITY; hi = -INFINITY;
    for (unsigned int b = threadIdx.x; b < gridDim.x; b += BLOCK) {
        lo = fminf(lo, __hip_atomic_load(&part[2 * b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        hi = fmaxf(hi, __hip_atomic_load(&part[2 * b + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    lo = wave_reduce_minmax<true>(lo);
    hi = wave_reduce_minmax<false>(hi);
    __syncthreads();
    if (lane == 0) { s_lo[wave] = lo; s_hi[wave] = hi; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < BLOCK / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
        RangeParams r;
        if (lo <= hi) {
            r.lo = lo; r.hi = hi;
            r.w = __fsub_rn(hi, lo);
            r.scale = (r.w > 0.0f) ? __fdiv_rn(fbins, r.w) : 0.0f;
        } else {   // no finite sample at all
            r.lo = NAN; r.hi = NAN; r.w = 0.0f; r.scale = 0.0f;
        }
        *rp = r;
        *done = 0u;
    }
}

// Caller-supplied range: same derived quantities, no pass over the data; zeroes the counters.
__global__ void k_set_range(RangeParams* rp, float lo, float hi, float fbins,
                            unsigned long long* counts, uint32_t bins, const unsigned int* gate)
{
    if (gate && __hip_atomic_load(gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < bins) counts[i] = 0ull;
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        RangeParams r;
        r.lo = lo; r.hi = hi;
        r.w = __fsub_rn(hi, lo);
        r.scale = (r.w > 0.0f) ? __fdiv_rn(fbins, r.w) : 0.0f;
        *rp = r;
    }
}

// ---------------------------------------------------------------------------
// kernel 2: histogram + entropy
// ---------------------------------------------------------------------------
template <typename T, int VEC, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_hist(
    const EntGroup grp, const RangeParams* __restrict__ rp, uint32_t bins,
    uint32_t bins_local, uint32_t rep_shift, unsigned long long* counts,
    unsigned int* done, edgc_entropy_result* res, const unsigned int* gate)
{
    if (gate && __hip_atomic_load(gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    extern __shared__ uint32_t h[];   // [bins_local << rep_shift], replica = lane & (R-1)
    const uint32_t bin_base = blockIdx.y * bins_local;
    const uint32_t local_n = min(bins_local, bins - bin_base);
    const uint32_t words = local_n << rep_shift;
    for (uint32_t i = threadIdx.x; i < words; i += BLOCK) h[i] = 0u;
    __syncthreads();

    const float lo = rp->lo, scale = rp->scale;
    const float fbins = static_cast<float>(bins);
    // largest float below the bin count: truncating a value clamped to [0, top] gives 0 .. bins - 1,
    // the same index as min(trunc(max(f, 0)), bins - 1)
    const float top = __uint_as_float(__float_as_uint(fbins) - 1u);
    const uint32_t rep = threadIdx.x & ((1u << rep_shift) - 1u);
    const bool whole = (gridDim.y == 1);      // one slice holds every bin
    uint32_t* const h_rep = h + rep;          // this lane's replica of bin b is h_rep[b << rep_shift]

    constexpr int U = 4;
    for (uint32_t ti = 0; ti < grp.count; ++ti) {
    const SampleGeom& geom = grp.geom[ti];
    const T* __restrict__ g = static_cast<const T*>(grp.base[ti]);
    const uint64_t per = (geom.n_items + gridDim.x - 1) / gridDim.x;      // one contiguous range per block
    const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * per;
    const uint64_t end = min(begin + per, geom.n_items);
    ItemCursor cur;
    cur.init(begin + threadIdx.x, BLOCK, geom.ipc);
    if constexpr (VEC > 1) {
        // Rounds of U whole items per thread, the next round's loads issued before the current round is
        // binned.  Every item before the buffer's last sampled chunk is whole (the chunk size is a multiple
        // of VEC), so these loads need no condition and stay in flight across the binning.
        const uint64_t fast_end = (geom.n_items >= geom.ipc) ? min(end, geom.n_items - geom.ipc) : 0;
        auto round_fits = [&]() { return cur.item + static_cast<uint64_t>(U - 1) * BLOCK < fast_end; };
        auto fetch_raw = [&](uint4 (&raw)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                raw[u] = *reinterpret_cast<const uint4*>(g + cur.elem0(geom, VEC));
                cur.advance(BLOCK, geom.ipc);
            }
        };
        auto bin_raw = [&](const uint4 (&raw)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float v[VEC];
                unpack_item<T, VEC>(raw[u], v);
#pragma unroll
                for (int p = 0; p < VEC; ++p) {
                    const float t = __fsub_rn(v[p], lo);
                    const float f = __builtin_amdgcn_fmed3f(__fmul_rn(t, scale), 0.0f, top);
                    atomicAdd(&h_rep[static_cast<uint32_t>(f) << rep_shift], finite_f32(v[p]) ? 1u : 0u);
                }
            }
        };
        // (measured on a 1e9-element buffer: with every element sampled 0.86 instead of 0.91 ms on fp32 and
        // 0.51 instead of 0.63 ms on bf16; on the 10 % sample, 256-byte runs 2.5 KB apart, 0.19 instead of
        // 0.15 ms, so strided samples keep the plain loop below)
        if (whole && geom.stride == 1 && round_fits()) {
            uint4 ra[U], rb[U];
            fetch_raw(ra);
            while (true) {
                if (!round_fits()) { bin_raw(ra); break; }
                fetch_raw(rb);
                bin_raw(ra);
                if (!round_fits()) { bin_raw(rb); break; }
                fetch_raw(ra);
                bin_raw(rb);
            }
        }
    }
    while (cur.item < end) {
        float v[U][VEC];
        uint32_t mask[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mask[u] = 0;
            if (cur.item < end) {
                const uint64_t i0 = cur.elem0(geom, VEC);
                if (i0 < geom.n) mask[u] = load_item<T, VEC>(g, i0, geom.n, v[u]);
            }
            cur.advance(BLOCK, geom.ipc);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (whole && mask[u] == (1u << VEC) - 1u) {
                // a whole item with every bin in this block's slice: no branch per element.  The index
                // of a non-finite value is some valid bin (the clamp maps NaN to 0) and it adds 0.
#pragma unroll
                for (int p = 0; p < VEC; ++p) {
                    const float x = v[u][p];
                    const float t = __fsub_rn(x, lo);
                    const float f = __builtin_amdgcn_fmed3f(__fmul_rn(t, scale), 0.0f, top);
                    atomicAdd(&h_rep[static_cast<uint32_t>(f) << rep_shift], finite_f32(x) ? 1u : 0u);
                }
                continue;
            }
#pragma unroll
            for (int p = 0; p < VEC; ++p) {
                if (!((mask[u] >> p) & 1u)) continue;
                const float x = v[u][p];
                if (!finite_f32(x)) continue;
                // bin = trunc((x - lo) * scale), each operation rounded on its own
                const float t = __fsub_rn(x, lo);
                float f = __fmul_rn(t, scale);
                f = fminf(fmaxf(f, 0.0f), fbins);          // also maps NaN (inf * 0) to 0
                const uint32_t b = min(static_cast<uint32_t>(f), bins - 1u);
                const uint32_t rel = b - bin_base;
                if (rel < local_n) atomicAdd(&h_rep[rel << rep_shift], 1u);
            }
        }
    }
    }
    __syncthreads();

    // fold the replicas and flush non-empty bins
    for (uint32_t i = threadIdx.x; i < local_n; i += BLOCK) {
        uint32_t s = 0;
        for (uint32_t r = 0; r < (1u << rep_shift); ++r) s += h[(i << rep_shift) | r];
        if (s) atomicAdd(&counts[bin_base + i], static_cast<unsigned long long>(s));
    }

    __shared__ bool s_last;
    __threadfence();                  // this thread's counter updates are visible device-wide
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int ticket = atomicAdd(done, 1u);
        s_last = (ticket == gridDim.x * gridDim.y - 1);
    }
    __syncthreads();
    if (!s_last) return;

    // last block: H = log2 n - (1/n) sum c log2 c   (== -sum p log2 p)
    __threadfence();
    finish_entropy<BLOCK>(counts, bins, rp, grp.n_sampled, res);
    if (threadIdx.x == 0) {
        *done = 0u;
        // every block of this grid has read the gate by now (each took its ticket after that)
        if (gate) *const_cast<unsigned int*>(gate) = 0u;
    }
}

// ---------------------------------------------------------------------------
// 65536 counters per block in LDS, as 16-bit fields (two per 32-bit word, 128 KiB, one block of
// 1024 threads per CU).  Two uses:
//  * fp32 samples on more than 16384 bins: the key of an element is its bin, and the sample is
//    binned in ONE read (32-bit counters cover 32768 bins per read);
//  * bf16 samples, whatever the number of bins: the key is the raw bit pattern.  A bf16 value is
//    one of 65536 patterns, and range, bin and finiteness are functions of the pattern alone, so
//    the sample is read ONCE, with no range pass before it, and the rest (range of the finite
//    sample, bin of every pattern by the same fp32 operations the binning kernel applies to
//    every element, entropy) is derived from the 65536 pattern counts.
// A field counts to 0x7fff; the add that takes it to 0x8000 or beyond sees that in the value the
// atomic returns, and that thread alone credits 32768 to the key's 64-bit global counter
// (`wide`) and takes 0x8000 off the field again.  A field could only carry into its neighbour if
// 32767 more increments reached it between those two LDS operations of one thread; the add that
// would do it sees 0xffff, and then the kernel raises `gate`, which lets the plain kernels queued
// behind on the stream redo the estimate (they return at once otherwise).
// At its end a block stores its fields as they stand to its own 128 KiB of `part16` (plain
// 16-byte stores: no atomics on global memory, of which 256 blocks x some thousand keys would be
// the larger part of a small estimate), and k_wide_reduce sums them.
// ---------------------------------------------------------------------------
constexpr int kWideBlock = 1024;
constexpr uint32_t kWideKeys = 65536;

__device__ __forceinline__ void field_add(uint32_t* h, unsigned long long* wide, uint32_t key, uint32_t k,
                                          uint32_t& overflow)
{
    const uint32_t sh = (key & 1u) << 4;
    const uint32_t old = atomicAdd(&h[key >> 1], k << sh);
    const uint32_t fld = (old >> sh) & 0xffffu;
    if (fld < 0x8000u && fld + k >= 0x8000u) {
        atomicAdd(&wide[key], 32768ull);
        atomicSub(&h[key >> 1], 0x8000u << sh);
    }
    if (fld + k > 0xffffu) overflow = 1u;
}

template <typename T, int VEC, bool PATTERN>
__global__ __launch_bounds__(kWideBlock) void k_wide_hist(
    const EntGroup grp, const RangeParams* __restrict__ rp, uint32_t bins, uint16_t* __restrict__ part16,
    unsigned long long* __restrict__ wide, unsigned int* gate, int raise_gate)
{
    static_assert(!PATTERN || sizeof(T) == 2, "the raw pattern is the key of 16-bit elements only");
    extern __shared__ uint32_t h[];   // [kWideKeys / 2]
    for (uint32_t i = threadIdx.x; i < kWideKeys / 2; i += kWideBlock) h[i] = 0u;
    __syncthreads();

    float lo = 0.0f, scale = 0.0f, top = 0.0f;
    if constexpr (!PATTERN) {
        lo = rp->lo; scale = rp->scale;
        const float fbins = static_cast<float>(bins);
        top = __uint_as_float(__float_as_uint(fbins) - 1u);     // largest float below the bin count
    }
    // bin = trunc((x - lo) * scale), each operation rounded on its own, clamped to [0, bins - 1]
    auto bin_of = [&](float x) {
        const float t = __fsub_rn(x, lo);
        return static_cast<uint32_t>(__builtin_amdgcn_fmed3f(__fmul_rn(t, scale), 0.0f, top));
    };

    uint32_t overflow = 0;
    constexpr int U = 4;
    for (uint32_t ti = 0; ti < grp.count; ++ti) {
        const SampleGeom& geom = grp.geom[ti];
        const T* __restrict__ g = static_cast<const T*>(grp.base[ti]);
        const uint64_t per = (geom.n_items + gridDim.x - 1) / gridDim.x;      // one contiguous range per block
        const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * per;
        const uint64_t end = min(begin + per, geom.n_items);
        ItemCursor cur;
        cur.init(begin + threadIdx.x, kWideBlock, geom.ipc);
        if constexpr (VEC > 1) {
            // rounds of U whole items per thread, the next round's loads in flight behind the current one
            const uint64_t fast_end = (geom.n_items >= geom.ipc) ? min(end, geom.n_items - geom.ipc) : 0;
            auto round_fits = [&]() { return cur.item + static_cast<uint64_t>(U - 1) * kWideBlock < fast_end; };
            auto fetch_raw = [&](uint4 (&raw)[U]) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    raw[u] = *reinterpret_cast<const uint4*>(g + cur.elem0(geom, VEC));
                    cur.advance(kWideBlock, geom.ipc);
                }
            };
            auto count_raw = [&](const uint4 (&raw)[U]) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (PATTERN) {
                        const uint32_t w[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t a = w[q] & 0xffffu, b = w[q] >> 16;
                            if (a == b) {                  // runs of equal values (zeros) in one add
                                field_add(h, wide, a, 2u, overflow);
                            } else {
                                field_add(h, wide, a, 1u, overflow);
                                field_add(h, wide, b, 1u, overflow);
                            }
                        }
                    } else {
                        float v[VEC];
                        unpack_item<T, VEC>(raw[u], v);
#pragma unroll
                        for (int q = 0; q < VEC; ++q)
                            field_add(h, wide, bin_of(v[q]), finite_f32(v[q]) ? 1u : 0u, overflow);
                    }
                }
            };
            if (round_fits()) {
                uint4 ra[U], rb[U];
                fetch_raw(ra);
                while (true) {
                    if (!round_fits()) { count_raw(ra); break; }
                    fetch_raw(rb);
                    count_raw(ra);
                    if (!round_fits()) { count_raw(rb); break; }
                    fetch_raw(ra);
                    count_raw(rb);
                }
            }
        }
        while (cur.item < end) {
            const uint64_t i0 = cur.elem0(geom, VEC);
#pragma unroll
            for (int q = 0; q < VEC; ++q) {
                if (i0 + q < geom.n) {
                    if constexpr (PATTERN) {
                        field_add(h, wide, g[i0 + q], 1u, overflow);
                    } else {
                        const float x = ElemTraits<T>::widen(g[i0 + q]);
                        if (finite_f32(x)) field_add(h, wide, bin_of(x), 1u, overflow);
                    }
                }
            }
            cur.advance(kWideBlock, geom.ipc);
        }
    }
    if (overflow || raise_gate) atomicOr(gate, 1u);   // raise_gate: the redo path under test
    __syncthreads();
    uint4* __restrict__ dst = reinterpret_cast<uint4*>(part16 + static_cast<size_t>(blockIdx.x) * kWideKeys);
    const uint4* h4 = reinterpret_cast<const uint4*>(h);
    for (uint32_t i = threadIdx.x; i < kWideKeys / 8; i += kWideBlock) dst[i] = h4[i];
}

// Sums the blocks' 16-bit fields and the 64-bit credits per key (one thread per key, 1024 keys per
// block), and the last block to finish turns the totals into the estimate.
//  fp32 (keys are bins): the totals are the histogram.
//  bf16 (keys are bit patterns): the blocks also reduce the range of the patterns that occur; the
//  last block bins the patterns' totals in LDS (slices of 16384 bins) and writes the histogram.
constexpr uint32_t kWideSliceBins = 16384;
constexpr size_t kWideReduceLds = 8 * kWideBlock * sizeof(uint32_t);      // the eight groups' sums

template <bool PATTERN>
__global__ __launch_bounds__(kWideBlock) void k_wide_reduce(
    const uint16_t* __restrict__ part16, uint32_t nblocks, unsigned long long* __restrict__ wide,
    unsigned long long* totals, uint32_t bins, int has_range, float range_lo, float range_hi,
    unsigned long long* counts, RangeParams* rp, float* part, unsigned int* done, const unsigned int* gate,
    unsigned long long n_sampled, edgc_entropy_result* res)
{
    extern __shared__ unsigned long long slice[];     // 32 KiB for the sums; PATTERN: [min(bins, kWideSliceBins)] as well
    constexpr uint32_t kMaxGrid = kWideKeys / kWideBlock;
    __shared__ bool s_last;
    __shared__ float s_lo[kWideBlock / 64], s_hi[kWideBlock / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t key = blockIdx.x * kWideBlock + threadIdx.x;
    // after a counter overflow the kernels behind redo the estimate, on counters that start at zero
    const bool redo = __hip_atomic_load(gate, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
    // per block: (lo, hi) of the patterns that occur, or (sum c log2 c, sum c) of its bins
    double* const part_d = reinterpret_cast<double*>(part);

    unsigned long long c = wide[key];
    if (c) wide[key] = 0ull;                          // zero between estimates
    {
        // The block's 1024 keys are 128 columns of eight 16-bit fields (one 16-byte load); each of its
        // eight groups of 128 threads sums every eighth block's fields, and the groups' sums meet in LDS.
        uint32_t* const red = reinterpret_cast<uint32_t*>(slice);          // [8][kWideBlock]
        const uint32_t col = threadIdx.x & 127u, grp = threadIdx.x >> 7;
        const uint4* __restrict__ src = reinterpret_cast<const uint4*>(part16 + blockIdx.x * kWideBlock) + col;
        constexpr size_t kRow = kWideKeys / 8;                             // 16-byte items per block's fields
        uint32_t sm[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};               // at most 32 blocks x 0xffff each
        for (uint32_t b = grp; b < nblocks; b += 64) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = (b + 8 * u < nblocks) ? src[static_cast<size_t>(b + 8 * u) * kRow] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                sm[0] += v[u].x & 0xffffu; sm[1] += v[u].x >> 16;
                sm[2] += v[u].y & 0xffffu; sm[3] += v[u].y >> 16;
                sm[4] += v[u].z & 0xffffu; sm[5] += v[u].z >> 16;
                sm[6] += v[u].w & 0xffffu; sm[7] += v[u].w >> 16;
            }
        }
        uint4* const dst = reinterpret_cast<uint4*>(red + grp * kWideBlock + col * 8);
        dst[0] = make_uint4(sm[0], sm[1], sm[2], sm[3]);
        dst[1] = make_uint4(sm[4], sm[5], sm[6], sm[7]);
        __syncthreads();
        uint32_t sum = 0;
#pragma unroll
        for (int gI = 0; gI < 8; ++gI) sum += red[gI * kWideBlock + threadIdx.x];
        c += sum;
        __syncthreads();                              // `slice` is used again by the last block
    }
    if constexpr (!PATTERN) {
        // the totals are the histogram; this block's share of the entropy sums goes with them
        if (key < bins) counts[key] = redo ? 0ull : c;
        double acc = 0.0, tot = 0.0;
        if (key < bins) entropy_term(c, acc, tot);
        block_sum_pair<kWideBlock>(acc, tot);
        if (threadIdx.x == 0) { part_d[2 * blockIdx.x] = acc; part_d[2 * blockIdx.x + 1] = tot; }
    } else {
        totals[key] = c;
        const float x = __uint_as_float(key << 16);
        float lo = INFINITY, hi = -INFINITY;
        if (c && finite_f32(x)) { lo = x; hi = x; }
        lo = wave_reduce_minmax<true>(lo);
        hi = wave_reduce_minmax<false>(hi);
        if (lane == 0) { s_lo[wave] = lo; s_hi[wave] = hi; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < kWideBlock / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
            part[2 * blockIdx.x]     = lo;            // lo > hi: none of this block's patterns occurs
            part[2 * blockIdx.x + 1] = hi;
        }
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int ticket = atomicAdd(done, 1u);
        s_last = (ticket == gridDim.x - 1);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();

    double acc = 0.0, tot = 0.0;
    if constexpr (!PATTERN) {
        if (threadIdx.x < gridDim.x) {
            acc = __hip_atomic_load(&part_d[2 * threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            tot = __hip_atomic_load(&part_d[2 * threadIdx.x + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    } else {
        // range of the finite sample from the blocks' partials, and the list of the blocks (of 1024
        // patterns) in which any pattern occurs: a dense gradient touches a few of the 64
        __shared__ float s_blo[kMaxGrid], s_bhi[kMaxGrid];
        __shared__ uint32_t s_list[kMaxGrid];
        __shared__ uint32_t s_nlist;
        __shared__ float s_range[2];
        if (threadIdx.x < gridDim.x) {
            s_blo[threadIdx.x] = __hip_atomic_load(&part[2 * threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_bhi[threadIdx.x] = __hip_atomic_load(&part[2 * threadIdx.x + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            float lo = INFINITY, hi = -INFINITY;
            uint32_t nl = 0;
            for (uint32_t b = 0; b < gridDim.x; ++b) {
                lo = fminf(lo, s_blo[b]); hi = fmaxf(hi, s_bhi[b]);
                if (s_blo[b] <= s_bhi[b]) s_list[nl++] = b;
            }
            s_nlist = nl;
            if (has_range) { lo = range_lo; hi = range_hi; }
            const float fbins = static_cast<float>(bins);
            RangeParams r;
            if (has_range || lo <= hi) {
                r.lo = lo; r.hi = hi;
                r.w = __fsub_rn(hi, lo);
                r.scale = (r.w > 0.0f) ? __fdiv_rn(fbins, r.w) : 0.0f;
            } else {   // no finite sample at all
                r.lo = NAN; r.hi = NAN; r.w = 0.0f; r.scale = 0.0f;
            }
            *rp = r;
            s_range[0] = r.lo; s_range[1] = r.scale;
        }
        __syncthreads();
        const float rlo = s_range[0], scale = s_range[1];
        const uint32_t nlist = s_nlist;
        const float fbins = static_cast<float>(bins);
        const float top = __uint_as_float(__float_as_uint(fbins) - 1u);   // largest float below the bin count
        for (uint32_t base = 0; base < bins; base += kWideSliceBins) {
            const uint32_t nb = min(kWideSliceBins, bins - base);
            for (uint32_t i = threadIdx.x; i < nb; i += kWideBlock) slice[i] = 0ull;
            __syncthreads();
            // eight of the listed blocks at a time: their loads (from the other blocks' stores, past this
            // CU's caches) are in flight together
            for (uint32_t j = 0; j < nlist; j += 8) {
                unsigned long long cp[8];
                uint32_t pp[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    pp[u] = s_list[min(j + u, nlist - 1)] * kWideBlock + threadIdx.x;
                    cp[u] = __hip_atomic_load(&totals[pp[u]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const float x = __uint_as_float(pp[u] << 16);
                    if (j + u < nlist && cp[u] && finite_f32(x)) {
                        // bin = trunc((x - lo) * scale), each operation rounded on its own, clamped to [0, bins - 1]
                        const float t = __fsub_rn(x, rlo);
                        const uint32_t bin =
                            static_cast<uint32_t>(__builtin_amdgcn_fmed3f(__fmul_rn(t, scale), 0.0f, top));
                        if (bin - base < nb) atomicAdd(&slice[bin - base], cp[u]);
                    }
                }
            }
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < nb; i += kWideBlock) {
                const unsigned long long cb = slice[i];
                counts[base + i] = redo ? 0ull : cb;
                entropy_term(cb, acc, tot);
            }
            __syncthreads();
        }
    }
    block_sum_pair<kWideBlock>(acc, tot);
    if (threadIdx.x == 0) {
        emit_result(acc, tot, bins, rp, n_sampled, res);
        *done = 0u;
    }
}

// ---------------------------------------------------------------------------
// sampled indices (same cursor as the kernels above)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_sample_indices(SampleGeom geom, uint64_t* __restrict__ idx,
                                                        uint64_t cap)
{
    const uint64_t G = static_cast<uint64_t>(gridDim.x) * 256;
    ItemCursor cur;
    cur.init(static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x, G, geom.ipc);
    const int vec = static_cast<int>(geom.vec);
    while (cur.item < geom.n_items) {
        const uint64_t i0 = cur.elem0(geom, vec);
        const uint64_t pos0 = cur.k * geom.chunk + static_cast<uint64_t>(cur.e) * vec;
        for (int p = 0; p < vec; ++p)
            if (i0 + p < geom.n && pos0 + p < cap) idx[pos0 + p] = i0 + p;
        cur.advance(G, geom.ipc);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
SampleGeom make_geom(const void* base, edgc_dtype dt, uint64_t n, uint64_t stride, uint32_t chunk,
                     uint64_t seed, uint64_t step, bool allow_vec)
{
    SampleGeom g{};
    const uint32_t elem = (dt == EDGC_F32) ? 4u : 2u;
    const uint32_t V = 16u / elem;
    const bool aligned = allow_vec && (reinterpret_cast<uintptr_t>(base) % 16u) == 0;
    g.n = n;
    g.stride = stride;
    g.slot = mix64(seed, step) % stride;
    g.chunk = chunk;
    if (stride == 1) {
        // every element is sampled whatever the chunk size: read it as long runs
        g.slot = 0;
        if (aligned) g.chunk = 4096;
    }
    const uint64_t total_chunks = (n + g.chunk - 1) / g.chunk;
    g.n_chunks = (g.slot < total_chunks) ? (total_chunks - g.slot + stride - 1) / stride : 0;
    g.n_sampled = 0;
    if (g.n_chunks) {
        const uint64_t last = g.slot + (g.n_chunks - 1) * stride;
        const uint64_t last_len = (n - last * g.chunk < g.chunk) ? n - last * g.chunk : g.chunk;
        g.n_sampled = (g.n_chunks - 1) * g.chunk + last_len;
    }
    g.vec = (aligned && g.chunk % V == 0) ? V : 1u;
    g.ipc = g.chunk / g.vec;
    g.n_items = g.n_chunks * g.ipc;
    return g;
}

static uint32_t grid_for(uint64_t n_items, int block, int per_thread, int max_blocks)
{
    uint64_t want = (n_items + static_cast<uint64_t>(block) * per_thread - 1) /
                    (static_cast<uint64_t>(block) * per_thread);
    if (want < 1) want = 1;
    if (want > static_cast<uint64_t>(max_blocks)) want = max_blocks;
    return static_cast<uint32_t>(want);
}

// The device memory an estimate works in beyond its inputs and outputs: the context's own
// allocations, or the file-scope array of the entry point that allocates nothing.
struct EntScratch {
    float*              mm_part;       // [2 * kMaxReduceBlocks] per-block (lo, hi)
    unsigned int*       done_counter;  // [4] last-block tickets (0..2) and the overflow gate (3), zero between calls
    uint16_t*           part16;        // [part16_blocks][65536] 16-bit counters per block, or null: plain kernels only
    uint32_t            part16_blocks;
    unsigned long long* wide;          // [65536] 64-bit credits per key, zero between calls
    unsigned long long* totals;        // [65536] counts per bf16 bit pattern
    unsigned long long* counts;        // histogram when the caller gives none
    void*               range;         // RangeParams
    void*               result_dev;    // edgc_entropy_result
};

template <typename T, int VEC>
static int run_entropy(edgc_ctx* ctx, const EntScratch& s, const EntGroup& g, uint32_t bins, const float* range,
                       uint64_t* counts_out, edgc_entropy_result* res, hipStream_t st)
{
    auto* counts = counts_out ? reinterpret_cast<unsigned long long*>(counts_out) : s.counts;
    auto* rp = static_cast<RangeParams*>(s.range);
    const float fbins = static_cast<float>(bins);

    const double sample_bytes = static_cast<double>(g.n_sampled) * sizeof(T);
    const bool small_sample = g.n_items <= static_cast<uint64_t>(kHistBlock) * 4 * ctx->num_cu * 2;
    // blocks a sample below 8 Mi items gets at most: 16 up to 1 Mi items; one per 32 Ki items from 2 Mi items on
    // (1e7 fp32 elements, 2.5 Mi items: 0.068 instead of 0.082 ms alone); between the two the launch shapes of
    // large samples (1e7 bf16 elements, 1.25 Mi items: 0.056 ms, with the cap 0.089)
    const uint64_t few_blocks = small_sample ? kSmallSampleBlocks
                              : (g.n_items >= (2ull << 20) ? (g.n_items >> 15) : ~0ull / (4 * kHistBlockFat));
    // One read into 16-bit counters per block (the kernels above), where the context has the memory
    // for the blocks' fields: every bf16 sample of some size (no range pass, any number of bins), and
    // fp32 samples on more bins than 32-bit counters hold in LDS at once.  The plain kernels follow on
    // the stream behind `gate` and return at once unless a 16-bit counter overflowed.
    const bool wide_ok = s.part16 != nullptr && ctx->tune_pattern != 0;
    // (measured on samples of a 1e9-element bf16 buffer, 4096 bins, one read against two passes: 1e7
    // elements 0.067 against 0.061 ms, 1e8 0.115 against 0.171, 1e9 0.57 against 0.85; on 65536 bins: 1e7
    // 0.103 against 0.155 ms, 1e9 0.61 against 1.87)
    const uint64_t pattern_min = static_cast<uint64_t>(ctx->tune_pattern_min);
    const bool by_pattern = sizeof(T) == 2 && wide_ok &&
                            (g.n_sampled >= pattern_min || (bins > 16384 && g.n_sampled >= pattern_min / 8));
    const bool by_wide_bins = sizeof(T) == 4 && wide_ok && bins > 16384 && bins <= kWideKeys;
    unsigned int* gate = (by_pattern || by_wide_bins) ? s.done_counter + 3 : nullptr;
    const uint32_t wide_blocks = grid_for(g.n_items, kWideBlock, 4, min(ctx->num_cu, static_cast<int>(s.part16_blocks)));
    if constexpr (sizeof(T) == 2) {
        if (by_pattern) {
            EDGC_LAUNCH(ctx, st, KID_WIDE_HIST, sample_bytes, 0.0,
                        k_wide_hist<T, VEC, true><<<wide_blocks, kWideBlock, kWideKeys * 2, st>>>(
                            g, rp, bins, s.part16, s.wide, gate, ctx->tune_pattern == 3 ? 1 : 0));
            const size_t lds = max(static_cast<size_t>(min(bins, kWideSliceBins)) * sizeof(unsigned long long),
                                   kWideReduceLds);
            EDGC_LAUNCH(ctx, st, KID_WIDE_REDUCE, 2.0 * kWideKeys * wide_blocks, 0.0,
                        k_wide_reduce<true><<<kWideKeys / kWideBlock, kWideBlock, lds, st>>>(
                            s.part16, wide_blocks, s.wide, s.totals, bins, range ? 1 : 0, range ? range[0] : 0.0f,
                            range ? range[1] : 0.0f, counts, rp, s.mm_part, s.done_counter + 2, gate,
                            g.n_sampled, res));
        }
    }
    if (range) {
        EDGC_LAUNCH(ctx, st, KID_SET_RANGE, 8.0 * bins, 0.0,
                    k_set_range<<<(bins + 255) / 256, 256, 0, st>>>(rp, range[0], range[1], fbins, counts,
                                                                     bins, by_pattern ? gate : nullptr));
    } else {
        // few blocks of four rounds of four 16-byte loads: the estimate runs beside the compressor's
        // streaming passes, and every block of it that takes a CU slot delays those (measured on the
        // bench workload: 16 items per thread cost 12 us of step time less than 4)
        if (g.n_items >= kBigSampleItems) {
            // a large sample: one block of 1024 threads per CU (1e8 fp32 elements out of 1e9: 0.08 instead
            // of 0.12 ms, bf16 0.05 instead of 0.08; every element of 1e9: 0.70 instead of 0.71 ms)
            const uint32_t gx = grid_for(g.n_items, kMMBlockFat, 16, ctx->num_cu);
            EDGC_LAUNCH(ctx, st, KID_MINMAX, sample_bytes, 0.0,
                        k_minmax<T, VEC, kMMBlockFat><<<gx, kMMBlockFat, 0, st>>>(g, s.mm_part, s.done_counter, rp,
                                                                                  fbins, counts, bins,
                                                                                  by_pattern ? gate : nullptr));
        } else {
            // a small sample (the 1 % sample of a transformer block's gradients, say) gets at most 16 blocks:
            // beside the compressor's passes it is the number of CU slots the estimate takes that costs step
            // time, not its own duration (hidden-5120 bf16 block at rank 128, 393 Ki items: 96 blocks of 16 items
            // per thread 1.241 ms per step, 12 blocks 1.207 ms, though the two kernels alone take 88 instead of 44 us)
            // (a 16 M-element sample of a 32-tensor stage, 4 Mi items: 983 and 491 blocks 6.90 ms per step and 87 + 123
            // us alone, 123 blocks each 6.82 ms and 69 + 82 us)
            const uint64_t few = static_cast<uint64_t>(kMMBlock) * few_blocks;
            const int mm_items = ctx->tune_ept > 0 ? 2 * ctx->tune_ept
                                                   : static_cast<int>(std::max<uint64_t>(16, (g.n_items + few - 1) / few));
            const uint32_t gx = grid_for(g.n_items, kMMBlock, mm_items, min(kMaxReduceBlocks, ctx->num_cu * 4));
            EDGC_LAUNCH(ctx, st, KID_MINMAX, sample_bytes, 0.0,
                        k_minmax<T, VEC, kMMBlock><<<gx, kMMBlock, 0, st>>>(g, s.mm_part, s.done_counter, rp,
                                                                            fbins, counts, bins,
                                                                            by_pattern ? gate : nullptr));
        }
    }

    if constexpr (sizeof(T) == 4) {
        if (by_wide_bins) {
            EDGC_LAUNCH(ctx, st, KID_WIDE_HIST, sample_bytes, 0.0,
                        k_wide_hist<T, VEC, false><<<wide_blocks, kWideBlock, kWideKeys * 2, st>>>(
                            g, rp, bins, s.part16, s.wide, gate, ctx->tune_pattern == 3 ? 1 : 0));
            EDGC_LAUNCH(ctx, st, KID_WIDE_REDUCE, 2.0 * kWideKeys * wide_blocks, 0.0,
                        k_wide_reduce<false><<<(bins + kWideBlock - 1) / kWideBlock, kWideBlock, kWideReduceLds, st>>>(
                            s.part16, wide_blocks, s.wide, s.totals, bins, 0, 0.0f, 0.0f, counts, rp, s.mm_part,
                            s.done_counter + 2, gate, g.n_sampled, res));
        }
    }

    // LDS plan: up to 64 KiB of 32-bit counters, replicated per lane where bins are few;
    // more than 16384 bins are covered in slices of 32768 (128 KiB), one slice per blockIdx.y
    // small samples get few blocks of few items each, and then fewer replicas so that zeroing
    // and folding the LDS histogram does not outweigh the sampling itself
    const bool small = small_sample;
    const uint32_t word_cap = small ? 4096u : 16384u;
    uint32_t bins_local = bins, rep_shift = 0;
    if (bins <= 16384) {
        while (rep_shift < 5 && (static_cast<uint64_t>(bins) << (rep_shift + 1)) <= word_cap) ++rep_shift;
    } else if (bins > 32768) {
        bins_local = 32768;
    }
    const uint32_t ny = (bins + bins_local - 1) / bins_local;
    const size_t lds = static_cast<size_t>(bins_local << rep_shift) * sizeof(uint32_t);
    // enough items per block that zeroing and flushing the LDS histogram stays small
    const uint64_t few_h = static_cast<uint64_t>(kHistBlock) * few_blocks;
    const int floor_items = small ? 8 : ((bins_local << rep_shift) > 16384 ? 64 : 16);
    const int per_thread = ctx->tune_ept > 0 ? ctx->tune_ept
                         : (g.n_items < kBigSampleItems
                                ? static_cast<int>(std::max<uint64_t>(floor_items, (g.n_items + few_h - 1) / few_h))
                                : floor_items);
    // One block of 1024 threads per CU when a histogram of more than 64 KiB leaves room for one block only
    // (1e9 fp32 elements on 65536 bins: 1.6 instead of 3.6 ms) and for samples of 8 Mi items or more (1e8
    // fp32 elements on 4096 bins: 0.13 instead of 0.18 ms; 1e9: 0.83 instead of 0.86 ms); two blocks of
    // 512 per CU otherwise (1e7 bf16 elements: 0.040 against 0.044 ms; two blocks of 1024: slower throughout)
    if (lds > 65536 || g.n_items >= kBigSampleItems) {
        const uint32_t gx = grid_for(g.n_items, kHistBlockFat, per_thread, ctx->num_cu);
        EDGC_LAUNCH(ctx, st, KID_HIST, sample_bytes * ny, 0.0,
                    k_hist<T, VEC, kHistBlockFat><<<dim3(gx, ny), kHistBlockFat, lds, st>>>(
                        g, rp, bins, bins_local, rep_shift, counts, s.done_counter + 1, res, gate));
    } else {
        const uint32_t gx = grid_for(g.n_items, kHistBlock, per_thread, ctx->num_cu * 2);
        EDGC_LAUNCH(ctx, st, KID_HIST, sample_bytes * ny, 0.0,
                    k_hist<T, VEC, kHistBlock><<<dim3(gx, ny), kHistBlock, lds, st>>>(
                        g, rp, bins, bins_local, rep_shift, counts, s.done_counter + 1, res, gate));
    }
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

int prepare_entropy_kernels(edgc_ctx* ctx)
{
    constexpr int lds = 32768 * 4;     // one slice of 32768 bins
    constexpr int wide_lds = kWideKeys * 2;
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wide_hist<uint16_t, 8, true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, wide_lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wide_hist<uint16_t, 1, true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, wide_lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wide_hist<float, 4, false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, wide_lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wide_hist<float, 1, false>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, wide_lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_wide_reduce<true>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize,
                                          static_cast<int>(kWideSliceBins * sizeof(unsigned long long))));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<float, 4, kHistBlock>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<float, 4, kHistBlockFat>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<float, 1, kHistBlock>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<float, 1, kHistBlockFat>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<uint16_t, 8, kHistBlock>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<uint16_t, 8, kHistBlockFat>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<uint16_t, 1, kHistBlock>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_hist<uint16_t, 1, kHistBlockFat>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    return EDGC_OK;
}

static int launch_entropy_on(edgc_ctx* ctx, const EntScratch& s, const EntGroup& g, edgc_dtype dt, uint32_t bins,
                             const float* range, edgc_entropy_result* out, uint64_t* counts_out, hipStream_t st)
{
    // the kernels are compiled for one vector width: every buffer of the group was given the same
    bool vec = true;
    for (uint32_t i = 0; i < g.count; ++i) vec = vec && g.geom[i].vec > 1;
    // Pinned (device-accessible) host memory takes the result straight from the kernel; any
    // other host memory gets it through a copy on the stream.
    auto* res = static_cast<edgc_entropy_result*>(s.result_dev);
    bool direct = false;
    hipPointerAttribute_t attr;
    if (reinterpret_cast<uintptr_t>(out) % alignof(edgc_entropy_result) == 0 &&
        hipPointerGetAttributes(&attr, out) == hipSuccess && attr.type == hipMemoryTypeHost &&
        attr.devicePointer != nullptr) {
        res = static_cast<edgc_entropy_result*>(attr.devicePointer);
        direct = true;
    } else {
        (void)hipGetLastError();      // pageable memory is reported as an error: not one here
    }
    int rc;
    if (dt == EDGC_F32)
        rc = vec ? run_entropy<float, 4>(ctx, s, g, bins, range, counts_out, res, st)
                 : run_entropy<float, 1>(ctx, s, g, bins, range, counts_out, res, st);
    else
        rc = vec ? run_entropy<uint16_t, 8>(ctx, s, g, bins, range, counts_out, res, st)
                 : run_entropy<uint16_t, 1>(ctx, s, g, bins, range, counts_out, res, st);
    if (rc != EDGC_OK || direct) return rc;
    EDGC_HIP_TRY(ctx, hipMemcpyAsync(out, s.result_dev, sizeof(edgc_entropy_result),
                                     hipMemcpyDeviceToHost, st));
    return EDGC_OK;
}

int launch_entropy(edgc_ctx* ctx, const EntGroup& g, edgc_dtype dt, uint32_t bins,
                   const float* range, edgc_entropy_result* out, uint64_t* counts_out, hipStream_t st)
{
    const Scratch& c = ctx->s;
    const EntScratch s{c.mm_part, c.done_counter, c.part16, c.part16_blocks, c.wide, c.totals,
                       c.counts, c.range, c.result_dev};
    return launch_entropy_on(ctx, s, g, dt, bins, range, out, counts_out, st);
}

// ---------------------------------------------------------------------------
// The estimate for callers that cannot allocate: its scratch is a file-scope device array, so
// nothing has to be allocated for it, by the library or by the caller.  Each GPU holds its own
// copy of the array at its own address; the address is looked up once per device, at the first
// edgc_create on that device (with that device current), and host code only ever uses that
// pointer, never the array's name.
// ---------------------------------------------------------------------------
constexpr size_t kStaticOffDone   = sizeof(float) * 2 * kMaxReduceBlocks;             // 32 KiB of (lo, hi) pairs
constexpr size_t kStaticOffRange  = kStaticOffDone + 256;
constexpr size_t kStaticOffResult = kStaticOffRange + 256;
constexpr size_t kStaticOffCounts = kStaticOffResult + 256;
constexpr size_t kStaticBytes     = kStaticOffCounts + sizeof(unsigned long long) * kStaticMaxBins;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
static unsigned char* g_static_scratch[kMaxDevices] = {};     // per device, set once

int resolve_static_scratch(edgc_ctx* ctx)
{
    const int dev = ctx->device;
    if (dev < 0 || dev >= kMaxDevices) return fail(ctx, EDGC_EINVAL, "device index beyond the static scratch table");
    if (g_static_scratch[dev]) return EDGC_OK;
    unsigned char* ptr = nullptr;
    EDGC_HIP_TRY(ctx, hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
    if (!ptr) return fail(ctx, EDGC_EHIP, "hipGetSymbolAddress returned a null address");
    // the tickets must start at zero; the array is zero-initialised when the code object is loaded
    // and every estimate leaves them at zero, but a process may have been interrupted mid-call
    EDGC_HIP_TRY(ctx, hipMemset(ptr + kStaticOffDone, 0, 256));
    EDGC_HIP_TRY(ctx, hipDeviceSynchronize());
    g_static_scratch[dev] = ptr;
    return EDGC_OK;
}

int launch_entropy_static(edgc_ctx* ctx, const EntGroup& g, edgc_dtype dt, uint32_t bins, const float* range,
                          edgc_entropy_result* out, uint64_t* counts_out, hipStream_t st)
{
    unsigned char* base = (ctx->device >= 0 && ctx->device < kMaxDevices) ? g_static_scratch[ctx->device] : nullptr;
    if (!base) return fail(ctx, EDGC_EHIP, "the static scratch of this device was not set up");
    const EntScratch s{reinterpret_cast<float*>(base),
                       reinterpret_cast<unsigned int*>(base + kStaticOffDone),
                       nullptr, 0u, nullptr, nullptr,     // no room for the blocks' 16-bit counters: plain kernels
                       reinterpret_cast<unsigned long long*>(base + kStaticOffCounts),
                       base + kStaticOffRange, base + kStaticOffResult};
    return launch_entropy_on(ctx, s, g, dt, bins, range, out, counts_out, st);
}

int launch_sample_indices(edgc_ctx* ctx, const SampleGeom& g, uint64_t* idx, uint64_t cap,
                          hipStream_t st)
{
    if (g.n_items == 0) return EDGC_OK;
    const uint32_t gx = grid_for(g.n_items, 256, 4, 65535);
    EDGC_LAUNCH(ctx, st, KID_SAMPLE_IDX, 8.0 * g.n_sampled, 0.0,
                k_sample_indices<<<gx, 256, 0, st>>>(g, idx, cap));
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

}  // namespace edgc
