// Q-pass  Q_partial[s] = D[row range s, :]^T P^[row range s, :]  (Sec. II-B: the second product of
// the PowerSGD step) for groups in which every tile is whole: rows a multiple of 64, columns a
// multiple of 256.  Same fragments and the same MFMA order as k_pass_q (compress.hip), hence the
// same bits; what differs is when the loads of D are issued.  k_pass_q requests a stage's 64 rows
// at the top of the stage, waits for them and multiplies: while a wave multiplies it has nothing in
// flight.  Here the two halves of a stage are converted to bf16 fragments one after the other, and
// as soon as a half's registers are free the same half of the NEXT stage is requested into them, so
// that a wave always has between half a stage and a whole stage of D in flight, at no cost in
// registers beyond the second pair of fragments.  Every load in the loop is unconditional (the last
// stage is peeled), which lets the compiler count what is in flight instead of waiting for all of it.
#include "compress_common.h"

namespace edgc {

template <int NP, int RT>
constexpr size_t pass_q_full_lds() { return static_cast<size_t>(2) * RT * 32 * (NP * 128 + 16); }

template <int NP, int RT, bool STREAM, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 2) void k_pass_q_full(const Group grp)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const float* __restrict__ D = ta.E;
    const __bf16* __restrict__ pt = static_cast<const __bf16*>(ta.pt);
    float* __restrict__ part = ta.part;
    const uint32_t m_pad = ta.m_pad, n = ta.n, stages_per_split = ta.d0, CB = ta.d1;
    constexpr int NT = 2;                            // columns per lane
    constexpr int RP = RT * 32;
    constexpr int ROWB = NP * 128 + 16;              // LDS bytes per factor column: 64 rows x NP planes + pad
    constexpr int TILE = RP * ROWB;
    constexpr int W = 32 * NT;
    constexpr int NSEG = RP * NP * 8;                // 16-byte segments of one P^ tile
    constexpr int NTH = 64 * WAVES;
    static_assert(NSEG % NTH == 0, "the P^ tile divides evenly among the threads");
    constexpr int PS = NSEG / NTH;
    extern __shared__ __attribute__((aligned(16))) unsigned char qlds[];   // 2 tiles

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t s = lid / CB, cb = lid % CB;
    const uint32_t jw0 = cb * WAVES * W + wave * W;
    const uint32_t st_begin = s * stages_per_split;
    const uint32_t st_end = min(m_pad / 64, st_begin + stages_per_split);
    // element offset of this lane inside a 16-row step: rows 8g .. 8g+7, columns jw0 + 2jl, +1 (fits 32 bits:
    // n < 2^28, checked on the host)
    const uint32_t off_l = 8u * g * n + jw0 + NT * jl;

    f32x16 acc[RT][NT];
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ct][t][v] = 0.0f;

    bf16x8 seg[PS];
    float dv[4][8][NT];

#define EDGC_QFULL_FETCH_PT(ST)                                                                           \
    {                                                                                                     \
        _Pragma("unroll") for (int p = 0; p < PS; ++p) {                                                  \
            const int it = tid + p * NTH;                                                                 \
            const int sg = it % 8, cp = it / 8, c = cp % RP, pl = cp / RP;                                \
            seg[p] = *reinterpret_cast<const bf16x8*>(                                                    \
                pt + (static_cast<size_t>(pl) * RP + c) * m_pad + (ST) * 64 + sg * 8);                    \
        }                                                                                                 \
    }
#define EDGC_QFULL_STORE_PT(BUF)                                                                          \
    {                                                                                                     \
        _Pragma("unroll") for (int p = 0; p < PS; ++p) {                                                  \
            const int it = tid + p * NTH;                                                                 \
            const int sg = it % 8, cp = it / 8, c = cp % RP, pl = cp / RP;                                \
            *reinterpret_cast<bf16x8*>(qlds + (BUF) * TILE + c * ROWB + pl * 128 + sg * 16) = seg[p];     \
        }                                                                                                 \
    }
    // the 16-row steps U0 and U0 + 1 of stage ST: rows 8g + q of each step, two adjacent columns
#define EDGC_QFULL_FETCH_D(ST, U0)                                                                        \
    {                                                                                                     \
        _Pragma("unroll") for (int uu = 0; uu < 2; ++uu) {                                                \
            _Pragma("unroll") for (int q = 0; q < 8; ++q) {                                               \
                const float* p_ = D + static_cast<uint64_t>((ST) * 64 + 16 * ((U0) + uu) + q) * n + off_l; \
                if constexpr (STREAM) {                                                                   \
                    const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(p_));           \
                    dv[(U0) + uu][q][0] = x.x; dv[(U0) + uu][q][1] = x.y;                                 \
                } else {                                                                                  \
                    const float2 x = *reinterpret_cast<const float2*>(p_);                                \
                    dv[(U0) + uu][q][0] = x.x; dv[(U0) + uu][q][1] = x.y;                                 \
                }                                                                                         \
            }                                                                                             \
        }                                                                                                 \
    }
    // one half of a stage: the 16-row steps 2H and 2H + 1
#define EDGC_QFULL_HALF(ST, MORE, H)                                                                      \
    {                                                                                                     \
        bf16x8 a[2][NT][NP];                                                                              \
        _Pragma("unroll") for (int uu = 0; uu < 2; ++uu) {                                                \
            _Pragma("unroll") for (int t = 0; t < NT; ++t) {                                              \
                float col8[8];                                                                            \
                _Pragma("unroll") for (int q = 0; q < 8; ++q) col8[q] = dv[2 * (H) + uu][q][t];           \
                pack8<NP>(col8, a[uu][t]);                                                                \
            }                                                                                             \
        }                                                                                                 \
        if constexpr (MORE) EDGC_QFULL_FETCH_D((ST) + 1, 2 * (H))                                         \
        _Pragma("unroll") for (int uu = 0; uu < 2; ++uu) {                                                \
            _Pragma("unroll") for (int ct = 0; ct < RT; ++ct) {                                           \
                bf16x8 b[NP];                                                                             \
                _Pragma("unroll") for (int p = 0; p < NP; ++p)                                            \
                    b[p] = *reinterpret_cast<const bf16x8*>(tile + (ct * 32 + jl) * ROWB + p * 128 + (2 * (H) + uu) * 32 + g * 16); \
                _Pragma("unroll") for (int t = 0; t < NT; ++t) acc[ct][t] = mma<NP>(a[uu][t], b, acc[ct][t]); \
            }                                                                                             \
        }                                                                                                 \
    }
#define EDGC_QFULL_STAGE(ST, MORE)                                                                        \
    {                                                                                                     \
        EDGC_QFULL_STORE_PT(buf)                                                                          \
        __syncthreads(); /* tile `buf` is complete; every wave is past its reads of stage ST-2 */         \
        if constexpr (MORE) EDGC_QFULL_FETCH_PT((ST) + 1)                                                 \
        const unsigned char* tile = qlds + buf * TILE;                                                    \
        EDGC_QFULL_HALF(ST, MORE, 0)                                                                      \
        EDGC_QFULL_HALF(ST, MORE, 1)                                                                      \
        buf ^= 1;                                                                                         \
    }

    if (st_begin < st_end) {
        EDGC_QFULL_FETCH_PT(st_begin)
        EDGC_QFULL_FETCH_D(st_begin, 0)
        EDGC_QFULL_FETCH_D(st_begin, 2)
        int buf = 0;
        uint32_t st = st_begin;
        for (; st + 1 < st_end; ++st) EDGC_QFULL_STAGE(st, true)
        EDGC_QFULL_STAGE(st, false)
    }
#undef EDGC_QFULL_STAGE
#undef EDGC_QFULL_HALF
#undef EDGC_QFULL_FETCH_D
#undef EDGC_QFULL_STORE_PT
#undef EDGC_QFULL_FETCH_PT

    // accumulator (ct, t, v) of lane l: column j = jw0 + NT*rho + t with rho = 8*(v/4) + 4*g + v%4,
    // factor column c = ct*32 + jl  ->  part[s][j][c]
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t j = jw0 + NT * (8 * (v / 4) + 4 * g + (v % 4)) + t;
                part[(static_cast<size_t>(s) * n + j) * RP + ct * 32 + jl] = acc[ct][t][v];
            }
}

// Whether a group meets what k_pass_q_full assumes (checked on the host before the launch).
bool pass_q_full_applies(const Group& g, edgc_dtype dt, int rt, uint32_t waves)
{
    if (waves != 4 && !(waves == 8 && rt >= 2)) return false;
    // fp32 above rank 64: the fragments of two planes leave no registers for a second pair
    if (dt != EDGC_BF16 && rt > 2) return false;
    for (uint32_t i = 0; i < g.count; ++i) {
        const TensorArgs& t = g.t[i];
        if (t.m % 64 || t.m_pad != t.m || t.n % (64 * waves)) return false;
        if (t.n >= (1u << 28)) return false;
        if (reinterpret_cast<uintptr_t>(t.E) % 8) return false;
    }
    return true;
}

template <int NP, int RT>
static hipError_t launch_qfull(const Group& g, uint32_t blocks, uint32_t waves, hipStream_t st)
{
    constexpr size_t lds = pass_q_full_lds<NP, RT>();
    static_assert(lds <= 64 * 1024, "fits the default dynamic LDS limit");
    if constexpr (RT >= 2) {
        if (waves == 8) {
            if (g.stream) k_pass_q_full<NP, RT, true, 8><<<blocks, 512, lds, st>>>(g);
            else k_pass_q_full<NP, RT, false, 8><<<blocks, 512, lds, st>>>(g);
            return hipGetLastError();
        }
    }
    if (g.stream) k_pass_q_full<NP, RT, true, 4><<<blocks, 256, lds, st>>>(g);
    else k_pass_q_full<NP, RT, false, 4><<<blocks, 256, lds, st>>>(g);
    return hipGetLastError();
}

hipError_t launch_pass_q_full(const Group& g, edgc_dtype dt, int rt, uint32_t blocks, uint32_t waves, hipStream_t st)
{
    if (dt == EDGC_BF16) {
        switch (rt) {
        case 1: return launch_qfull<1, 1>(g, blocks, waves, st);
        case 2: return launch_qfull<1, 2>(g, blocks, waves, st);
        default: return launch_qfull<1, 4>(g, blocks, waves, st);
        }
    }
    switch (rt) {
    case 1: return launch_qfull<2, 1>(g, blocks, waves, st);
    default: return launch_qfull<2, 2>(g, blocks, waves, st);
    }
}

}  // namespace edgc
