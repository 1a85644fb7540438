// Reconstruction M^ = P^ Q^T -> grad_out (Sec. IV-D-1, T_decompress; Sec. VII error feedback in
// its deferred form: the residual buffer keeps D and this pass only writes M^) for groups in
// which every tile is whole: rows a multiple of the block's rows, columns a multiple of 64,
// output aligned for two-column stores.  Same fragments and the same MFMA order as
// k_decompress (compress.hip), hence the same bits; what differs is the code shape:
//   - no edge paths and a single loop, which brings the kernel from ~200 to ~120 registers
//     (three to four waves per SIMD: at rank 128 the pass does 128 flop per byte it writes and
//     needs its MFMA, conversion and store phases of different waves to overlap);
//   - WAVES x 32 rows per block share one staged tile of Q rows (eight waves: half the L2
//     traffic and half the conversion work per output byte);
//   - the Q tile is double-buffered in LDS: one block barrier per 64-column stage.
#include "compress_common.h"

namespace edgc {

template <int NP, int RT>
constexpr size_t decompress_full_lds() { return static_cast<size_t>(2) * 64 * (NP * RT * 32 * 2 + 16); }

template <int NP, int RT, int WAVES>
__global__ __launch_bounds__(64 * WAVES, (NP == 2 && RT == 4) ? 2 : ((RT == 4 && WAVES == 4) ? 3 : 4)) void k_decompress_full(const Group grp)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const float* __restrict__ P = ta.P;
    const float* __restrict__ Q = ta.Q;
    void* __restrict__ out_ = ta.out;
    const uint64_t ldo = ta.ldo;
    const uint32_t ldp = ta.ldp, ldq = ta.ldq, n = ta.n, r = grp.r;
    const uint32_t stages_per_split = ta.d0, JS = ta.d1;
    constexpr bool OUT_BF16 = (NP == 1);
    constexpr int KT = RT * 2;                        // 16-wide k blocks over the padded rank
    constexpr int RP = RT * 32;
    constexpr int ROWB = NP * RP * 2 + 16;            // LDS bytes per Q row
    constexpr int TILE = 64 * ROWB;
    constexpr int NTH = 64 * WAVES;
    constexpr int PQ = 64 * (RP / 4) / NTH;           // float4 items of a Q stage per thread
    static_assert(64 * (RP / 4) % NTH == 0, "the Q stage divides evenly among the threads");
    extern __shared__ __attribute__((aligned(16))) unsigned char dlds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t js = lid % JS, rb = lid / JS;
    const uint32_t row0 = rb * (32 * WAVES) + wave * 32;

    // A-fragments: row row0 + jl of P^, k = kb*16 + 8g .. +8
    bf16x8 a[KT][NP];
    {
        const uint32_t row = row0 + jl;
#pragma unroll
        for (int kb = 0; kb < KT; ++kb) {
            float v[8];
            const uint32_t c0 = kb * 16 + 8 * g;
            if (c0 + 8 <= r) {
                const float4 x = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0);
                const float4 y = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0 + 4);
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (c0 + e < r) ? P[static_cast<size_t>(row) * ldp + c0 + e] : 0.0f;
            }
            pack8<NP>(v, a[kb]);
        }
    }

    const uint32_t st_begin = js * stages_per_split;
    const uint32_t st_end = min(n / 64, st_begin + stages_per_split);   // st_begin < n / 64 by the launch's split

    float qv[PQ][4];
    // rank columns from ldq on are masked when the tile is staged: any address inside the row will do
#define EDGC_DFULL_FETCH_Q(ST)                                                                            \
    _Pragma("unroll") for (int p = 0; p < PQ; ++p) {                                                      \
        const int idx = tid + p * NTH;                                                                    \
        const int jj = idx / (RP / 4), c4 = (idx % (RP / 4)) * 4;                                         \
        const uint32_t cc = min(static_cast<uint32_t>(c4), ldq - 4u);                                     \
        const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>((ST) * 64 + jj) * ldq + cc); \
        qv[p][0] = q.x; qv[p][1] = q.y; qv[p][2] = q.z; qv[p][3] = q.w;                                   \
    }
    // row 2*jl + ct of the stage goes to LDS row ct*32 + jl: a lane's two tiles are adjacent columns
#define EDGC_DFULL_STAGE_Q(BUF)                                                                           \
    _Pragma("unroll") for (int p = 0; p < PQ; ++p) {                                                      \
        const int idx = tid + p * NTH;                                                                    \
        const int jj = idx / (RP / 4), c4 = (idx % (RP / 4)) * 4;                                         \
        float m4[4];                                                                                      \
        _Pragma("unroll") for (int e = 0; e < 4; ++e)                                                     \
            m4[e] = (static_cast<uint32_t>(c4 + e) < r) ? qv[p][e] : 0.0f;                                \
        bf16x4 w[NP];                                                                                     \
        pack4<NP>(m4, w);                                                                                 \
        const int lrow = (jj & 1) * 32 + (jj >> 1);                                                       \
        _Pragma("unroll") for (int q = 0; q < NP; ++q)                                                    \
            *reinterpret_cast<bf16x4*>(dlds + (BUF) * TILE + lrow * ROWB + q * (RP * 2) + c4 * 2) = w[q]; \
    }
#define EDGC_DFULL_PRODUCT_STORE(ST, BUF)                                                                 \
    {                                                                                                     \
        f32x16 acc[2];                                                                                    \
        _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) {                                                \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[ct][v] = 0.0f;                             \
            _Pragma("unroll") for (int kb = 0; kb < KT; ++kb) {                                           \
                bf16x8 b[NP];                                                                             \
                _Pragma("unroll") for (int p = 0; p < NP; ++p)                                            \
                    b[p] = *reinterpret_cast<const bf16x8*>(dlds + (BUF) * TILE + (ct * 32 + jl) * ROWB + p * (RP * 2) + kb * 32 + g * 16); \
                acc[ct] = mma<NP>(a[kb], b, acc[ct]);                                                     \
            }                                                                                             \
        }                                                                                                 \
        const uint32_t col = (ST) * 64 + 2 * jl;                                                          \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                  \
            const uint32_t row = row0 + 8 * (v / 4) + 4 * g + (v % 4);                                    \
            if constexpr (OUT_BF16) {                                                                     \
                const bf16x2 hh = {static_cast<__bf16>(acc[0][v]), static_cast<__bf16>(acc[1][v])};       \
                bf16x2* po = reinterpret_cast<bf16x2*>(static_cast<__bf16*>(out_) + static_cast<size_t>(row) * ldo + col); \
                __builtin_nontemporal_store(hh, po);   /* not read again here: past the caches */         \
            } else {                                                                                      \
                const vf2 q2 = {acc[0][v], acc[1][v]};                                                    \
                vf2* po = reinterpret_cast<vf2*>(static_cast<float*>(out_) + static_cast<size_t>(row) * ldo + col); \
                __builtin_nontemporal_store(q2, po);                                                      \
            }                                                                                             \
        }                                                                                                 \
    }

    // stage st multiplies from buffer (st - st_begin) & 1 while the next stage's rows are converted
    // into the other buffer and the rows after that are in flight
    EDGC_DFULL_FETCH_Q(st_begin)
    EDGC_DFULL_STAGE_Q(0)
    if (st_begin + 1 < st_end) EDGC_DFULL_FETCH_Q(st_begin + 1)
    int buf = 0;
    uint32_t st = st_begin;
    for (; st + 2 < st_end; ++st) {
        __syncthreads();      // tile `buf` is complete; every wave is past its reads of the other one
        EDGC_DFULL_STAGE_Q(buf ^ 1)
        EDGC_DFULL_FETCH_Q(st + 2)
        EDGC_DFULL_PRODUCT_STORE(st, buf)
        buf ^= 1;
    }
    if (st + 1 < st_end) {
        __syncthreads();
        EDGC_DFULL_STAGE_Q(buf ^ 1)
        EDGC_DFULL_PRODUCT_STORE(st, buf)
        buf ^= 1;
        ++st;
    }
    __syncthreads();
    EDGC_DFULL_PRODUCT_STORE(st, buf)
#undef EDGC_DFULL_PRODUCT_STORE
#undef EDGC_DFULL_STAGE_Q
#undef EDGC_DFULL_FETCH_Q
}

// What k_decompress_full assumes of every tensor of the group, checked on the host; `rows` are
// the rows of a block.
static bool group_is_full(const Group& g, uint32_t rows, uint32_t esz)
{
    if (!g.defer) return false;
    for (uint32_t i = 0; i < g.count; ++i) {
        const TensorArgs& t = g.t[i];
        if (!t.out || t.m % rows || t.n % 64 || t.ldo % 2 || t.ldq < 4) return false;
        if (reinterpret_cast<uintptr_t>(t.out) % (2 * esz)) return false;
    }
    return true;
}

bool decompress_full_applies(const Group& g, edgc_dtype dt, uint32_t waves)
{
    return group_is_full(g, 32 * waves, dt == EDGC_BF16 ? 2u : 4u);
}

template <int NP, int RT>
static hipError_t launch_dfull(const Group& g, uint32_t blocks, uint32_t waves, hipStream_t st)
{
    constexpr size_t lds = decompress_full_lds<NP, RT>();
    if (waves == 8) k_decompress_full<NP, RT, 8><<<blocks, 512, lds, st>>>(g);
    else k_decompress_full<NP, RT, 4><<<blocks, 256, lds, st>>>(g);
    return hipGetLastError();
}

hipError_t launch_decompress_full(const Group& g, edgc_dtype dt, int rt, uint32_t blocks, uint32_t waves,
                                  hipStream_t st)
{
#define EDGC_DISPATCH(NP_)                                           \
    switch (rt) {                                                    \
    case 1: return launch_dfull<NP_, 1>(g, blocks, waves, st);       \
    case 2: return launch_dfull<NP_, 2>(g, blocks, waves, st);       \
    default: return launch_dfull<NP_, 4>(g, blocks, waves, st);      \
    }
    if (dt == EDGC_BF16) { EDGC_DISPATCH(1) }
    EDGC_DISPATCH(2)
#undef EDGC_DISPATCH
}

template <int NP, int RT>
static hipError_t allow_lds_dfull()
{
    constexpr int lds = static_cast<int>(decompress_full_lds<NP, RT>());
    if (lds <= 64 * 1024) return hipSuccess;
    const void* fns[2] = {reinterpret_cast<const void*>(&k_decompress_full<NP, RT, 4>),
                          reinterpret_cast<const void*>(&k_decompress_full<NP, RT, 8>)};
    for (const void* f : fns) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t prepare_decompress_full()
{
    return allow_lds_dfull<2, 4>();     // 2 x 64 x 528 bytes
}

}  // namespace edgc
