// P-pass with the deferred subtraction (Sec. II-B power iteration, Sec. III-B / VII error
// feedback) for groups in which every tile is whole: every matrix has a multiple of 128 rows
// and of 64 columns, a residual from the step before, and alignment for 8-byte accesses.
// This is the steady state of a training run at the layer shapes of transformer blocks, and
// the case the rank-128 sweep is bound by.  Arithmetic, fragment order and results are those of
// k_pass_p_deferred (compress.hip):
//   E = D_prev - round(P^_prev Q_prev^T),  D = G + E (written back),  P_partial[s] = D Q_prev
// What differs is the code shape: one loop with unconditional loads (so the compiler can count
// the loads in flight and a wait for the Q rows leaves the G / D_prev loads behind them
// alone), no ragged-edge paths, and two block barriers per stage: the D tile a wave multiplies
// is the one it wrote itself, which needs no block barrier.  Without the edge paths the 4 x 16
// accumulators of 128 factor columns fit beside a 64-column stage, so ranks above 64 keep the
// 8-byte accesses of the 64-column form (bf16 gradients: 54 KB of LDS, two blocks per CU).
#include "compress_common.h"

namespace edgc {

template <int NP, int RT, int WAVES>
constexpr size_t pass_p_full_lds()
{
    return static_cast<size_t>(64) * (NP * RT * 32 * 2 + 16) + static_cast<size_t>(RT * 32 + 32 * WAVES) * (NP * 128 + 16);
}

// WAVES x 32 rows per block share the staged Q tiles (two LDS layouts per stage): eight waves halve that
// staging work per row.
template <int NP, int RT, bool STREAM, bool QLATE, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 2) void k_pass_p_deferred_full(const Group grp)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    using GT = typename GradElem<NP>::type;
    const GT* __restrict__ G = static_cast<const GT*>(ta.G);
    float* __restrict__ E = ta.E;
    const float* __restrict__ Q = ta.Q;
    const float* __restrict__ P = ta.P;
    float* __restrict__ part = ta.part;
    const uint64_t ldg = ta.ldg;
    const uint32_t ldq = ta.ldq, ldp = ta.ldp, m = ta.m, n = ta.n, r = grp.r, kper = ta.d0, S = ta.d1;
    constexpr bool ROUND_BF16 = (NP == 1);
    // QLATE: the next stage's Q rows are requested only after this stage's G / D_prev registers
    // have been consumed (fewer registers live at once, less time for the Q rows to arrive).
    constexpr int KT = RT * 2, RP = RT * 32;
    constexpr int ROWQ = NP * RP * 2 + 16;            // LDS bytes per Q row, [column][rank]
    constexpr int ROWB = NP * 128 + 16;               // LDS bytes per row of 64 columns
    constexpr int NTH = 64 * WAVES;
    static_assert(32 * (RP / 4) % NTH == 0, "the Q stage divides evenly among the threads");
    constexpr int PQ = 32 * (RP / 4) / NTH;           // Q-stage items per thread: 2 rows x 4 ranks each
    extern __shared__ __attribute__((aligned(16))) unsigned char plds[];
    unsigned char* ldsQ = plds;                       // 64 x ROWQ
    unsigned char* ldsT = ldsQ + 64 * ROWQ;           // RP x ROWB: Q^T
    unsigned char* ldsA = ldsT + RP * ROWB;           // 32 WAVES x ROWB: D, 32 rows per wave

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t s = lid % S, rb = lid / S;
    const uint32_t row0 = rb * (32 * WAVES) + wave * 32;
    const uint32_t k_begin = s * kper;
    const uint32_t k_end = min(n, k_begin + kper);
    const uint32_t n_st = (k_end - k_begin) / 64;     // whole stages only (the host checks)
    // per-lane element offsets inside a 32-row x 64-column stage (both fit 32 bits: n, ldg < 2^28)
    const uint32_t off_d = 4u * g * n + 2u * jl;
    const uint32_t off_g = 4u * g * static_cast<uint32_t>(ldg) + 2u * jl;

    // A-fragments of P^_prev: row row0 + jl, k = kb*16 + 8g .. +8
    bf16x8 a[KT][NP];
#pragma unroll
    for (int kb = 0; kb < KT; ++kb) {
        float v[8];
        const uint32_t row = row0 + jl, c0 = kb * 16 + 8 * g;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0.0f;
        if (c0 + 8 <= r) {
            const float4 x = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0);
            const float4 y = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0 + 4);
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (c0 + e < r) v[e] = P[static_cast<size_t>(row) * ldp + c0 + e];
        }
        pack8<NP>(v, a[kb]);
    }

    float qv[PQ][2][4];
    float dv[16][2], gv[16][NP];      // bf16 gradients: the pair of columns as loaded, widened where used

    f32x16 accp[RT];
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) accp[ct][v] = 0.0f;

    // Q rows of a stage: item (jp, c4) holds rows 2jp and 2jp+1 (two adjacent columns of the
    // matrix), ranks c4 .. c4+3; lanes run along jp.  Rank columns from ldq on are masked when
    // the tile is staged: any address inside the row will do for them.
#define EDGC_FULL_FETCH_Q(ST)                                                                             \
    {                                                                                                     \
        const uint32_t col0 = k_begin + (ST) * 64;                                                        \
        _Pragma("unroll") for (int p = 0; p < PQ; ++p) {                                                  \
            const int idx = tid + p * NTH;                                                                \
            const int jp = idx & 31, c4 = (idx >> 5) * 4;                                                 \
            const uint32_t cc = min(static_cast<uint32_t>(c4), ldq - 4u);                                 \
            _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                               \
                const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(col0 + 2 * jp + h) * ldq + cc); \
                qv[p][h][0] = q.x; qv[p][h][1] = q.y; qv[p][h][2] = q.z; qv[p][h][3] = q.w;               \
            }                                                                                             \
        }                                                                                                 \
    }
    // G and D_prev of this lane's 16 rows x 2 adjacent columns
#define EDGC_FULL_FETCH_DG(ST)                                                                            \
    {                                                                                                     \
        const uint32_t col0 = k_begin + (ST) * 64;                                                        \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                  \
            const uint32_t rowu = row0 + 8 * (v / 4) + (v % 4);                                           \
            const GT* pg = G + (static_cast<uint64_t>(rowu) * ldg + col0) + off_g;                        \
            const float* pd = E + (static_cast<uint64_t>(rowu) * n + col0) + off_d;                       \
            if constexpr (NP == 2) {                                                                      \
                const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(pg));               \
                gv[v][0] = x.x; gv[v][1] = x.y;                                                           \
            } else {                                                                                      \
                gv[v][0] = __uint_as_float(__builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(pg))); \
            }                                                                                             \
            if constexpr (STREAM) {                                                                       \
                const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(pd));               \
                dv[v][0] = x.x; dv[v][1] = x.y;                                                           \
            } else {                                                                                      \
                const float2 x = *reinterpret_cast<const float2*>(pd);                                    \
                dv[v][0] = x.x; dv[v][1] = x.y;                                                           \
            }                                                                                             \
        }                                                                                                 \
    }
    // ... into LDS twice: [column][rank] (row 2jp + h at LDS row h*32 + jp, so that a lane of the
    // first product ends up with two adjacent columns) and [rank][column], there as 32-bit words
    // of two adjacent columns
#define EDGC_FULL_STAGE_Q()                                                                               \
    _Pragma("unroll") for (int p = 0; p < PQ; ++p) {                                                      \
        const int idx = tid + p * NTH;                                                                    \
        const int jp = idx & 31, c4 = (idx >> 5) * 4;                                                     \
        uint32_t w[2][2][NP];                                                                             \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                                   \
            float m4[4];                                                                                  \
            _Pragma("unroll") for (int e = 0; e < 4; ++e)                                                 \
                m4[e] = (static_cast<uint32_t>(c4 + e) < r) ? qv[p][h][e] : 0.0f;                         \
            pack_pair<NP>(m4[0], m4[1], w[h][0]);                                                         \
            pack_pair<NP>(m4[2], m4[3], w[h][1]);                                                         \
        }                                                                                                 \
        _Pragma("unroll") for (int q = 0; q < NP; ++q) {                                                  \
            _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                               \
                const u32x2 two = {w[h][0][q], w[h][1][q]};                                               \
                *reinterpret_cast<u32x2*>(ldsQ + (h * 32 + jp) * ROWQ + q * (RP * 2) + c4 * 2) = two;     \
            }                                                                                             \
            _Pragma("unroll") for (int e2 = 0; e2 < 2; ++e2) {                                            \
                const uint32_t lo = __builtin_amdgcn_perm(w[1][e2][q], w[0][e2][q], 0x05040100u);         \
                const uint32_t hi = __builtin_amdgcn_perm(w[1][e2][q], w[0][e2][q], 0x07060302u);         \
                *reinterpret_cast<uint32_t*>(ldsT + (c4 + 2 * e2) * ROWB + q * 128 + jp * 4) = lo;        \
                *reinterpret_cast<uint32_t*>(ldsT + (c4 + 2 * e2 + 1) * ROWB + q * 128 + jp * 4) = hi;    \
            }                                                                                             \
        }                                                                                                 \
    }
    // M^_prev of the stage from LDS, as the decompress formed it; E = D_prev - M^_prev, D = G + E:
    // to the residual buffer and, as bf16 planes, to the wave's own LDS rows; then D Q.
#define EDGC_FULL_STAGE(ST, MORE)                                                                         \
    {                                                                                                     \
        __syncthreads(); /* every wave is past its reads of the previous stage's Q tiles */               \
        EDGC_FULL_STAGE_Q()                                                                               \
        __syncthreads();                                                                                  \
        if constexpr (MORE && !QLATE) EDGC_FULL_FETCH_Q((ST) + 1)                                         \
        f32x16 acc[2];                                                                                    \
        _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) {                                                \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[ct][v] = 0.0f;                             \
            _Pragma("unroll") for (int kb = 0; kb < KT; ++kb) {                                           \
                bf16x8 b[NP];                                                                             \
                _Pragma("unroll") for (int p = 0; p < NP; ++p)                                            \
                    b[p] = *reinterpret_cast<const bf16x8*>(ldsQ + (ct * 32 + jl) * ROWQ + p * (RP * 2) + kb * 32 + g * 16); \
                acc[ct] = mma<NP>(a[kb], b, acc[ct]);                                                     \
            }                                                                                             \
        }                                                                                                 \
        {                                                                                                 \
            const uint32_t col0 = k_begin + (ST) * 64;                                                    \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                              \
                const int rl = 8 * (v / 4) + (v % 4);                                                     \
                float w0 = acc[0][v], w1 = acc[1][v];                                                     \
                if constexpr (ROUND_BF16) {                                                               \
                    w0 = static_cast<float>(static_cast<__bf16>(w0));                                     \
                    w1 = static_cast<float>(static_cast<__bf16>(w1));                                     \
                }                                                                                         \
                float g0, g1;                                                                             \
                if constexpr (NP == 1) {                                                                  \
                    const uint32_t bits = __float_as_uint(gv[v][0]);                                      \
                    g0 = __uint_as_float(bits << 16); g1 = __uint_as_float(bits & 0xffff0000u);           \
                } else {                                                                                  \
                    g0 = gv[v][0]; g1 = gv[v][NP - 1];                                                    \
                }                                                                                         \
                const float d0 = g0 + (dv[v][0] - w0), d1 = g1 + (dv[v][1] - w1);                         \
                float* pd = E + (static_cast<uint64_t>(row0 + rl) * n + col0) + off_d;                    \
                *reinterpret_cast<float2*>(pd) = make_float2(d0, d1);                                     \
                uint32_t w[NP];                                                                           \
                pack_pair<NP>(d0, d1, w);                                                                 \
                _Pragma("unroll") for (int q = 0; q < NP; ++q)                                            \
                    *reinterpret_cast<uint32_t*>(ldsA + (wave * 32 + rl + 4 * g) * ROWB + q * 128 + jl * 4) = w[q]; \
            }                                                                                             \
        }                                                                                                 \
        if constexpr (MORE) EDGC_FULL_FETCH_DG((ST) + 1)                                                  \
        if constexpr (MORE && QLATE) EDGC_FULL_FETCH_Q((ST) + 1)                                          \
        /* the wave reads back the rows it has just written: its own LDS accesses stay in order */        \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                            \
        __builtin_amdgcn_wave_barrier();                                                                  \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");                                            \
        const unsigned char* pa = ldsA + (wave * 32 + jl) * ROWB + g * 16;                                \
        const unsigned char* pb = ldsT + jl * ROWB + g * 16;                                              \
        _Pragma("unroll") for (int kb = 0; kb < 4; ++kb) {                                                \
            bf16x8 af[NP];                                                                                \
            _Pragma("unroll") for (int q = 0; q < NP; ++q)                                                \
                af[q] = *reinterpret_cast<const bf16x8*>(pa + q * 128 + kb * 32);                         \
            _Pragma("unroll") for (int ct = 0; ct < RT; ++ct) {                                           \
                bf16x8 b[NP];                                                                             \
                _Pragma("unroll") for (int q = 0; q < NP; ++q)                                            \
                    b[q] = *reinterpret_cast<const bf16x8*>(pb + ct * 32 * ROWB + q * 128 + kb * 32);     \
                accp[ct] = mma<NP>(af, b, accp[ct]);                                                      \
            }                                                                                             \
        }                                                                                                 \
    }

    if (n_st) {
        EDGC_FULL_FETCH_Q(0)
        EDGC_FULL_FETCH_DG(0)
        uint32_t st = 0;
        for (; st + 1 < n_st; ++st) EDGC_FULL_STAGE(st, true)
        EDGC_FULL_STAGE(st, false)
    }
#undef EDGC_FULL_STAGE
#undef EDGC_FULL_STAGE_Q
#undef EDGC_FULL_FETCH_DG
#undef EDGC_FULL_FETCH_Q

    // partial P of this k-range: part[s][row][c], c over the padded rank
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = row0 + 8 * (v / 4) + 4 * g + (v % 4);
            part[(static_cast<size_t>(s) * m + row) * RP + ct * 32 + jl] = accp[ct][v];
        }
}

// Whether a group meets what k_pass_p_deferred_full assumes (checked on the host before the
// launch; the grid decomposition d0 = columns per split is a multiple of 64 by construction).
template <int NP>
static bool group_is_full(const Group& g, uint32_t waves)
{
    using GT = typename GradElem<NP>::type;
    if (!g.defer) return false;
    for (uint32_t i = 0; i < g.count; ++i) {
        const TensorArgs& t = g.t[i];
        if (t.e_zero || !t.G) return false;
        if (t.m % (32 * waves) || t.n % 64 || t.ldg % 2) return false;
        if (t.ldg >= (1ull << 28) || t.n >= (1u << 28)) return false;
        if (t.ldq < 4) return false;
        if (reinterpret_cast<uintptr_t>(t.G) % (2 * sizeof(GT)) || reinterpret_cast<uintptr_t>(t.E) % 8) return false;
    }
    return true;
}

bool pass_p_full_applies(const Group& g, edgc_dtype dt, int rt, uint32_t waves)
{
    if (waves != 4 && !(waves == 8 && rt >= 2)) return false;
    if (dt == EDGC_BF16) return group_is_full<1>(g, waves);
    // fp32 gradients above rank 64: eight waves only (138 KB of LDS, one block per CU)
    if (rt > 2 && waves != 8) return false;
    return group_is_full<2>(g, waves);
}

template <int NP, int RT, int WAVES>
static hipError_t launch_full_w(const Group& g, uint32_t blocks, bool qlate, hipStream_t st)
{
    constexpr size_t lds = pass_p_full_lds<NP, RT, WAVES>();
    constexpr int NTH = 64 * WAVES;
    if (g.stream) {
        if (qlate) k_pass_p_deferred_full<NP, RT, true, true, WAVES><<<blocks, NTH, lds, st>>>(g);
        else k_pass_p_deferred_full<NP, RT, true, false, WAVES><<<blocks, NTH, lds, st>>>(g);
    } else {
        if (qlate) k_pass_p_deferred_full<NP, RT, false, true, WAVES><<<blocks, NTH, lds, st>>>(g);
        else k_pass_p_deferred_full<NP, RT, false, false, WAVES><<<blocks, NTH, lds, st>>>(g);
    }
    return hipGetLastError();
}

template <int NP, int RT>
static hipError_t launch_full(const Group& g, uint32_t blocks, bool qlate, uint32_t waves, hipStream_t st)
{
    if constexpr (RT >= 2) {
        if (waves == 8) return launch_full_w<NP, RT, 8>(g, blocks, qlate, st);
    }
    return launch_full_w<NP, RT, 4>(g, blocks, qlate, st);
}

hipError_t launch_pass_p_full(const Group& g, edgc_dtype dt, int rt, uint32_t blocks, bool qlate, uint32_t waves,
                              hipStream_t st)
{
    if (dt == EDGC_BF16) {
        switch (rt) {
        case 1: return launch_full<1, 1>(g, blocks, qlate, waves, st);
        case 2: return launch_full<1, 2>(g, blocks, qlate, waves, st);
        default: return launch_full<1, 4>(g, blocks, qlate, waves, st);
        }
    }
    switch (rt) {
    case 1: return launch_full<2, 1>(g, blocks, qlate, waves, st);
    case 2: return launch_full<2, 2>(g, blocks, qlate, waves, st);
    default: return launch_full_w<2, 4, 8>(g, blocks, qlate, st);
    }
}

template <int NP, int RT, int WAVES>
static hipError_t allow_lds_full()
{
    constexpr int lds = static_cast<int>(pass_p_full_lds<NP, RT, WAVES>());
    if (lds <= 64 * 1024) return hipSuccess;
    const void* fns[4] = {reinterpret_cast<const void*>(&k_pass_p_deferred_full<NP, RT, true, true, WAVES>),
                          reinterpret_cast<const void*>(&k_pass_p_deferred_full<NP, RT, true, false, WAVES>),
                          reinterpret_cast<const void*>(&k_pass_p_deferred_full<NP, RT, false, true, WAVES>),
                          reinterpret_cast<const void*>(&k_pass_p_deferred_full<NP, RT, false, false, WAVES>)};
    for (const void* f : fns) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t prepare_pass_p_full()
{
    hipError_t e = allow_lds_full<2, 2, 4>();
    if (e == hipSuccess) e = allow_lds_full<1, 4, 4>();
    if (e == hipSuccess) e = allow_lds_full<1, 2, 8>();
    if (e == hipSuccess) e = allow_lds_full<1, 4, 8>();
    if (e == hipSuccess) e = allow_lds_full<2, 2, 8>();
    if (e == hipSuccess) e = allow_lds_full<2, 4, 8>();
    return e;
}

}  // namespace edgc
