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

// ---------------------------------------------------------------------------
// kernel 1: range of the finite sample
// ---------------------------------------------------------------------------
template <typename T, int VEC, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_minmax(const EntGroup grp,
                                                     float* __restrict__ part,
                                                     unsigned int* done, RangeParams* rp,
                                                     float fbins, unsigned long long* counts,
                                                     uint32_t bins)
{
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
                            unsigned long long* counts, uint32_t bins)
{
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
    unsigned int* done, edgc_entropy_result* res)
{
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
    __shared__ double s_a[BLOCK / 64], s_b[BLOCK / 64];
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
    double acc = 0.0, tot = 0.0;
    for (uint32_t i = threadIdx.x; i < bins; i += BLOCK) {
        const unsigned long long c =
            __hip_atomic_load(&counts[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (c) {
            const double d = static_cast<double>(c);
            acc += d * log2(d);
            tot += d;
        }
    }
    acc = wave_sum_f64(acc);
    tot = wave_sum_f64(tot);
    if ((threadIdx.x & 63) == 0) { s_a[threadIdx.x >> 6] = acc; s_b[threadIdx.x >> 6] = tot; }
    __syncthreads();
    if (threadIdx.x == 0) {
        acc = 0.0; tot = 0.0;
        for (int w = 0; w < BLOCK / 64; ++w) { acc += s_a[w]; tot += s_b[w]; }
        edgc_entropy_result r;
        r.lo = rp->lo; r.hi = rp->hi;
        r.n_sampled = grp.n_sampled;
        // every finite element of the sample was counted in exactly one bin (values outside a caller's
        // range in the edge bins), so what the bins do not hold is the non-finite part; the counts are
        // integers below 2^53, their sum in fp64 is exact
        r.n_nonfinite = grp.n_sampled - static_cast<unsigned long long>(tot);
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
    unsigned int*       done_counter;  // [2] last-block tickets, zero between calls
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
    if (range) {
        EDGC_LAUNCH(ctx, st, KID_SET_RANGE, 8.0 * bins, 0.0,
                    k_set_range<<<(bins + 255) / 256, 256, 0, st>>>(rp, range[0], range[1], fbins, counts,
                                                                     bins));
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
                                                                                  fbins, counts, bins));
        } else {
            const uint32_t gx = grid_for(g.n_items, kMMBlock, 16, min(kMaxReduceBlocks, ctx->num_cu * 4));
            EDGC_LAUNCH(ctx, st, KID_MINMAX, sample_bytes, 0.0,
                        k_minmax<T, VEC, kMMBlock><<<gx, kMMBlock, 0, st>>>(g, s.mm_part, s.done_counter, rp,
                                                                            fbins, counts, bins));
        }
    }

    // LDS plan: up to 64 KiB of 32-bit counters, replicated per lane where bins are few;
    // more than 16384 bins are covered in slices of 32768 (128 KiB), one slice per blockIdx.y
    // small samples get few blocks of few items each, and then fewer replicas so that zeroing
    // and folding the LDS histogram does not outweigh the sampling itself
    const bool small = g.n_items <= static_cast<uint64_t>(kHistBlock) * 4 * ctx->num_cu * 2;
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
    const int per_thread = small ? 8 : ((bins_local << rep_shift) > 16384 ? 64 : 16);
    // One block of 1024 threads per CU when a histogram of more than 64 KiB leaves room for one block only
    // (1e9 fp32 elements on 65536 bins: 1.6 instead of 3.6 ms) and for samples of 8 Mi items or more (1e8
    // fp32 elements on 4096 bins: 0.13 instead of 0.18 ms; 1e9: 0.83 instead of 0.86 ms); two blocks of
    // 512 per CU otherwise (1e7 bf16 elements: 0.040 against 0.044 ms; two blocks of 1024: slower throughout)
    if (lds > 65536 || g.n_items >= kBigSampleItems) {
        const uint32_t gx = grid_for(g.n_items, kHistBlockFat, per_thread, ctx->num_cu);
        EDGC_LAUNCH(ctx, st, KID_HIST, sample_bytes * ny, 0.0,
                    k_hist<T, VEC, kHistBlockFat><<<dim3(gx, ny), kHistBlockFat, lds, st>>>(
                        g, rp, bins, bins_local, rep_shift, counts, s.done_counter + 1, res));
    } else {
        const uint32_t gx = grid_for(g.n_items, kHistBlock, per_thread, ctx->num_cu * 2);
        EDGC_LAUNCH(ctx, st, KID_HIST, sample_bytes * ny, 0.0,
                    k_hist<T, VEC, kHistBlock><<<dim3(gx, ny), kHistBlock, lds, st>>>(
                        g, rp, bins, bins_local, rep_shift, counts, s.done_counter + 1, res));
    }
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

int prepare_entropy_kernels(edgc_ctx* ctx)
{
    constexpr int lds = 32768 * 4;     // one slice of 32768 bins
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
    const EntScratch s{c.mm_part, c.done_counter, c.counts, c.range, c.result_dev};
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
