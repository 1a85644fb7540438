// Rank-r low-rank compressor with error feedback on gfx950 (Sec. II-B: power
// iteration + orthogonalisation; Sec. III-B / VII: error feedback).
//
//   k_pass_p        D = G + E_old (written back), P_partial = D Q    (split over columns)
//   k_reduce_gram   P = sum of partials; per-block Gram P^T P in fp64
//   k_gram_sum      Gram = sum of the per-block Grams (only when there are many)
//   k_chol          scaled Cholesky of the Gram in fp64, inverse factor R^-1
//   k_apply         P^ = P R^-1 (fp64), plus a transposed bf16 operand copy of P^
//   k_pass_q        Q_partial = D^T P^                                (split over rows)
//   k_reduce_q      Q = sum of partials
//   k_decompress    M^ = P^ Q^T -> grad_out, E_new = D - M^
//   k_pass_p_deferred   the P-pass when the residual buffer kept D of the step before instead of E
//                   (batched calls, deferred = 1): E = D_prev - P^_prev Q_prev^T is formed on the
//                   way and k_decompress then only writes M^
//   k_pass_p_deferred_narrow   the same above rank 64 (32-column stages)
//
// All contractions run on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.
// bf16 gradients use one bf16 plane per operand (operands rounded to nearest
// even); fp32 gradients use two planes x = hi + lo (hi = bf16(x), lo =
// bf16(x - hi)) and three MFMAs per product (hi*hi, hi*lo, lo*hi), which keeps
// ~17 bits per operand.  The passes are HBM-bound (2r/(b+8), r/2 and r/6 flop
// per byte), so the matrix is streamed exactly once per pass with 16-byte
// accesses and everything else (factors, partials) stays in L2 / LDS.
//
// Every kernel works on a list of tensors (Group): its grid is the concatenation
// of the tensors' block ranges, so all gradients of a pipeline stage go through
// each pass in ONE launch; a single-tensor call is a list of one.
//
// MFMA 32x32x16 operand layout (64 lanes): lane l supplies A[i = l%32][k = 8*(l/32) .. +8]
// and B[k = 8*(l/32) .. +8][j = l%32]; accumulator register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].
#include "compress_common.h"

#include <algorithm>
#include <math.h>
#include <type_traits>

namespace edgc {

// ---------------------------------------------------------------------------
// seeded N(0,1) start of Q
// ---------------------------------------------------------------------------
__global__ void k_init_q(float* Q, uint32_t n, uint32_t ldq, uint32_t c0, uint32_t c1, uint64_t seed)
{
    const uint32_t w = c1 - c0;
    const uint64_t t = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= static_cast<uint64_t>(n) * w) return;
    const uint32_t j = static_cast<uint32_t>(t / w), c = c0 + static_cast<uint32_t>(t % w);
    const uint64_t k = (static_cast<uint64_t>(j) << 32) | c;
    const uint64_t z1 = mix64(seed, 2ull * k), z2 = mix64(seed, 2ull * k + 1ull);
    const double u1 = (static_cast<double>(z1 >> 11) + 0.5) * (1.0 / 9007199254740992.0);
    const double u2 = static_cast<double>(z2 >> 11) * (1.0 / 9007199254740992.0);
    Q[static_cast<size_t>(j) * ldq + c] =
        static_cast<float>(sqrt(-2.0 * log(u1)) * cos(6.28318530717958647692 * u2));
}

// ---------------------------------------------------------------------------
// P-pass:  D = G + E_old,  P_partial[s] = D[:, k-range s] * Q[k-range s, :]
// Block: 4 waves x 32 rows = 128 rows; k-step of 64 columns.
// ---------------------------------------------------------------------------
template <int NP, bool VECOK>
__device__ __forceinline__ void load_grad4(const typename GradElem<NP>::type* __restrict__ G,
                                           uint64_t ldg, uint32_t row, uint32_t col, uint32_t m,
                                           uint32_t col_end, float (&v)[4])
{
    v[0] = v[1] = v[2] = v[3] = 0.0f;
    if (G == nullptr || row >= m || col >= col_end) return;   // null gradient: D is re-read as it stands
    const auto* p = G + static_cast<uint64_t>(row) * ldg + col;
    if (VECOK && col + 4 <= col_end) {
        if constexpr (NP == 2) {
            const float4 q = *reinterpret_cast<const float4*>(p);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
            const uint2 q = *reinterpret_cast<const uint2*>(p);
            v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
            v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < col_end) {
                if constexpr (NP == 2) v[e] = p[e];
                else v[e] = bf16_bits_widen(p[e]);
            }
    }
}

template <bool VECOK>
__device__ __forceinline__ void load_f32x4(const float* __restrict__ base, uint64_t ld, uint32_t row,
                                           uint32_t col, uint32_t rows, uint32_t col_end, float (&v)[4])
{
    v[0] = v[1] = v[2] = v[3] = 0.0f;
    if (row >= rows || col >= col_end) return;
    const float* p = base + static_cast<uint64_t>(row) * ld + col;
    if (VECOK && col + 4 <= col_end) {
        const float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) if (col + e < col_end) v[e] = p[e];
    }
}

template <bool VECOK>
__device__ __forceinline__ void store_f32x4(float* __restrict__ base, uint64_t ld, uint32_t row,
                                            uint32_t col, uint32_t rows, uint32_t col_end,
                                            const float (&v)[4])
{
    if (row >= rows || col >= col_end) return;
    float* p = base + static_cast<uint64_t>(row) * ld + col;
    if (VECOK && col + 4 <= col_end) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) if (col + e < col_end) p[e] = v[e];
    }
}

// 16-byte streaming load that does not pollute the caches (the matrix is read once per pass)
typedef float vf4 __attribute__((ext_vector_type(4)));
typedef uint32_t vu2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void ld_stream4(const float* __restrict__ p, float (&v)[4])
{
    const vf4 q = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(p));
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
}
__device__ __forceinline__ void ld_stream4(const uint16_t* __restrict__ p, float (&v)[4])
{
    const vu2 q = __builtin_nontemporal_load(reinterpret_cast<const vu2*>(p));
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
}

template <int NP, int RT, bool VECOK>
__global__ __launch_bounds__(256) void k_pass_p(const Group grp)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const auto* __restrict__ G = static_cast<const typename GradElem<NP>::type*>(ta.G);
    float* __restrict__ E = ta.E;
    const float* __restrict__ Q = ta.Q;
    float* __restrict__ part = ta.part;
    const uint64_t ldg = ta.ldg;
    const uint32_t ldq = ta.ldq, m = ta.m, n = ta.n, r = grp.r, kper = ta.d0, S = ta.d1;
    const bool e_zero = ta.e_zero != 0;
    constexpr int BK  = 64;                        // k elements per step: 256 B (fp32) per row
    constexpr int ROWB = NP * 128 + 16;            // LDS bytes per tile row: planes + pad
    constexpr int RPP = 16;                        // rows per load pass (16 threads per row)
    constexpr int PA  = 128 / RPP;                 // load passes for the 128-row tile
    constexpr int RP  = RT * 32;                   // padded rank
    constexpr int NQI = RP * (BK / 8);             // Q-tile work items: one column x 8 k each
    constexpr int PQ  = (NQI + 255) / 256;

    __shared__ __attribute__((aligned(16))) unsigned char lds[(128 + RP) * ROWB];
    unsigned char* ldsA = lds;
    unsigned char* ldsB = lds + 128 * ROWB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t s = lid % S, rb = lid / S;
    const uint32_t row0 = rb * 128;
    const uint32_t k_begin = s * kper;
    const uint32_t k_end = min(n, k_begin + kper);
    const bool rows_full = row0 + 128 <= m;

    const int a_row = tid >> 4, a_col = (tid & 15) * 4;

    float d[PA][4];
    float qv[PQ][8];

    // FULL: the whole 128 x 64 tile is inside the matrix and vector accesses are allowed
    auto fetch = [&](uint32_t k0, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            const uint32_t row = row0 + p * RPP + a_row, col = k0 + a_col;
            float g[4] = {0.f, 0.f, 0.f, 0.f}, e[4] = {0.f, 0.f, 0.f, 0.f};
            if constexpr (FULL) {
                if (G) ld_stream4(G + static_cast<uint64_t>(row) * ldg + col, g);
                if (!e_zero) {
                    const float* pe = E + static_cast<uint64_t>(row) * n + col;
                    if (grp.stream) {
                        ld_stream4(pe, e);
                    } else {                                  // the residual may still be cached: keep it so
                        const float4 q4 = *reinterpret_cast<const float4*>(pe);
                        e[0] = q4.x; e[1] = q4.y; e[2] = q4.z; e[3] = q4.w;
                    }
                }
            } else {
                load_grad4<NP, VECOK>(G, ldg, row, col, m, k_end, g);
                if (!e_zero) load_f32x4<VECOK>(E, n, row, col, m, k_end, e);
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) d[p][x] = g[x] + e[x];
        }
        // Q tile: lane = factor column (256 B contiguous per wave load), 8 consecutive k per item
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int it = tid + p * 256;
            const uint32_t c = it % RP, k8 = it / RP;
            const bool live = it < NQI && c < r;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const uint32_t k = k0 + k8 * 8 + kk;
                qv[p][kk] = (live && (FULL || k < k_end)) ? Q[static_cast<uint64_t>(k) * ldq + c] : 0.0f;
            }
        }
    };
    auto commit = [&](uint32_t k0, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            const uint32_t row = row0 + p * RPP + a_row, col = k0 + a_col;
            if constexpr (FULL)
                *reinterpret_cast<float4*>(E + static_cast<uint64_t>(row) * n + col) =
                    make_float4(d[p][0], d[p][1], d[p][2], d[p][3]);
            else
                store_f32x4<VECOK>(E, n, row, col, m, k_end, d[p]);
            bf16x4 w[NP];
            pack4<NP>(d[p], w);
#pragma unroll
            for (int q = 0; q < NP; ++q)
                *reinterpret_cast<bf16x4*>(ldsA + (p * RPP + a_row) * ROWB + q * 128 + a_col * 2) = w[q];
        }
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int it = tid + p * 256;
            if (it < NQI) {
                const uint32_t c = it % RP, k8 = it / RP;
                bf16x8 w[NP];
                pack8<NP>(qv[p], w);
#pragma unroll
                for (int q = 0; q < NP; ++q)
                    *reinterpret_cast<bf16x8*>(ldsB + c * ROWB + q * 128 + k8 * 16) = w[q];
            }
        }
    };
    auto tile_full = [&](uint32_t k0) { return VECOK && rows_full && k0 + BK <= k_end; };
    using T = std::true_type;
    using F = std::false_type;

    f32x16 acc[RT];
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[ct][v] = 0.0f;

    if (k_begin < k_end) { if (tile_full(k_begin)) fetch(k_begin, T{}); else fetch(k_begin, F{}); }
    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
        __syncthreads();                         // previous step's LDS reads are done
        // D back to the residual buffer, operands into LDS
        if (tile_full(k0)) commit(k0, T{}); else commit(k0, F{});
        __syncthreads();
        if (k0 + BK < k_end) {                   // next tile's loads fly during the MFMAs
            if (tile_full(k0 + BK)) fetch(k0 + BK, T{}); else fetch(k0 + BK, F{});
        }
        const unsigned char* pa = ldsA + (wave * 32 + (lane & 31)) * ROWB + (lane >> 5) * 16;
        const unsigned char* pb = ldsB + (lane & 31) * ROWB + (lane >> 5) * 16;
#pragma unroll
        for (int kb = 0; kb < BK / 16; ++kb) {
            bf16x8 a[NP];
#pragma unroll
            for (int q = 0; q < NP; ++q) a[q] = *reinterpret_cast<const bf16x8*>(pa + q * 128 + kb * 32);
#pragma unroll
            for (int ct = 0; ct < RT; ++ct) {
                bf16x8 b[NP];
#pragma unroll
                for (int q = 0; q < NP; ++q)
                    b[q] = *reinterpret_cast<const bf16x8*>(pb + ct * 32 * ROWB + q * 128 + kb * 32);
                acc[ct] = mma<NP>(a, b, acc[ct]);
            }
        }
    }

    // partial P of this k-range: part[s][row][c], c over the padded rank
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = row0 + wave * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
            if (row < m)
                part[(static_cast<size_t>(s) * m + row) * RP + ct * 32 + (lane & 31)] = acc[ct][v];
        }
}

// ---------------------------------------------------------------------------
// Orthonormalisation of P (m x r): Cholesky-QR with the Gram matrix in fp64.
//   k_reduce_gram  P = sum of the column-split partials (split order); Gram tiles of the
//                  block's rows on v_mfma_f64_16x16x4_f64 (upper-triangle 16x16 tiles)
//   k_gram_sum     sum of the per-block Gram tiles (many blocks, 8 loads in flight)
//   k_chol         scaled Cholesky W = D^-1 L L^T D^-1 and R^-1 = D L^-T, one block
//   k_apply        P^ = P R^-1 on fp64 MFMA, fp32 result in place + bf16 operand copy
// fp64 MFMA 16x16x4 layout: lane l supplies A[i = l%16][k = l/16] and B[k = l/16][j = l%16];
// accumulator v of lane l holds D[i = l/16 + 4v][j = l%16].
// ---------------------------------------------------------------------------
typedef double f64x4 __attribute__((ext_vector_type(4)));

// t-th tile of the upper triangle of a T x T tile grid, row-major: (ta <= tb)
__host__ __device__ inline void tri_tile(int t, int T, int& ta, int& tb)
{
    ta = 0;
    int len = T;
    while (t >= len) { t -= len; ++ta; --len; }
    tb = ta + t;
}

template <int T16>
__global__ __launch_bounds__(256) void k_reduce_gram(const Group grp, uint32_t RP)
{
    const TensorArgs& ta_ = grp.t[locate(grp, blockIdx.x)];
    const float* __restrict__ part = ta_.part;
    float* __restrict__ P = ta_.P;
    double* __restrict__ gram_part = ta_.gram_part;
    const uint32_t S = ta_.sp, m = ta_.m, r = grp.r, ldp = ta_.ldp, chunks_per_block = ta_.d0;
    const uint32_t bid = blockIdx.x - ta_.first;
    constexpr int CW = 16 * T16;
    constexpr int LD = CW + 16;                      // floats; 4 rows x 16 columns per read: 2-way at worst
    constexpr int NTILE = T16 * (T16 + 1) / 2;
    constexpr int TPW = (NTILE + 3) / 4;             // Gram tiles per wave
    __shared__ __attribute__((aligned(16))) float Ps[64 * LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    int ta[TPW], tb[TPW];
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + 4 * q;
        tri_tile(t < NTILE ? t : 0, T16, ta[q], tb[q]);
    }
    f64x4 acc[TPW];
#pragma unroll
    for (int q = 0; q < TPW; ++q) acc[q] = f64x4{0.0, 0.0, 0.0, 0.0};

    const uint32_t total_chunks = (m + 63) / 64;
    const uint32_t ch_begin = bid * chunks_per_block;
    const uint32_t ch_end = min(total_chunks, ch_begin + chunks_per_block);
    const size_t sstride = static_cast<size_t>(m) * RP;
    for (uint32_t ch = ch_begin; ch < ch_end; ++ch) {
        const uint32_t row0 = ch * 64;
        __syncthreads();                             // previous chunk's Gram reads are done
        // the sums of all T16 items of a thread advance together, DEP splits at a time, so that
        // DEP * T16 independent 16-byte loads are in flight (the order of the additions per element
        // is the split order, whatever the grouping)
        float4 v[T16];
        const float* src[T16];
#pragma unroll
        for (int it = 0; it < T16; ++it) {
            const int idx = tid + 256 * it;
            const int i = idx / (CW / 4), c4 = (idx % (CW / 4)) * 4;
            const uint32_t row = min(row0 + i, m - 1);       // rows past the end are loaded but not used
            v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            src[it] = part + static_cast<size_t>(row) * RP + c4;
        }
        constexpr int DEP = T16 >= 4 ? 2 : 4;            // splits per round
        uint32_t sp = 0;
        for (; sp + DEP <= S; sp += DEP) {
            float4 x[DEP][T16];
#pragma unroll
            for (int u = 0; u < DEP; ++u)
#pragma unroll
                for (int it = 0; it < T16; ++it)
                    x[u][it] = *reinterpret_cast<const float4*>(src[it] + (sp + u) * sstride);
#pragma unroll
            for (int u = 0; u < DEP; ++u)
#pragma unroll
                for (int it = 0; it < T16; ++it) {
                    v[it].x += x[u][it].x; v[it].y += x[u][it].y; v[it].z += x[u][it].z; v[it].w += x[u][it].w;
                }
        }
        for (; sp < S; ++sp) {
#pragma unroll
            for (int it = 0; it < T16; ++it) {
                const float4 x0 = *reinterpret_cast<const float4*>(src[it] + sp * sstride);
                v[it].x += x0.x; v[it].y += x0.y; v[it].z += x0.z; v[it].w += x0.w;
            }
        }
#pragma unroll
        for (int it = 0; it < T16; ++it) {
            const int idx = tid + 256 * it;
            const int i = idx / (CW / 4), c4 = (idx % (CW / 4)) * 4;
            const uint32_t row = row0 + i;
            if (row < m) {
                // partial columns >= r are exact zeros (the Q tile is masked in the P-pass)
                float* dst = P + static_cast<size_t>(row) * ldp + c4;
                if (static_cast<uint32_t>(c4) + 4 <= r) {
                    *reinterpret_cast<float4*>(dst) = v[it];
                } else {
                    if (static_cast<uint32_t>(c4) < r) dst[0] = v[it].x;
                    if (static_cast<uint32_t>(c4) + 1 < r) dst[1] = v[it].y;
                    if (static_cast<uint32_t>(c4) + 2 < r) dst[2] = v[it].z;
                }
            } else {
                v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            *reinterpret_cast<float4*>(Ps + i * LD + c4) = v[it];
        }
        __syncthreads();
        const float* pk = Ps + (lane >> 4) * LD + (lane & 15);
#pragma unroll 4
        for (int k0 = 0; k0 < 64; k0 += 4) {
#pragma unroll
            for (int q = 0; q < TPW; ++q) {
                // rows from column tile tb, columns from column tile ta: the tile below the diagonal
                const double a = static_cast<double>(pk[k0 * LD + 16 * tb[q]]);
                const double b = static_cast<double>(pk[k0 * LD + 16 * ta[q]]);
                acc[q] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[q], 0, 0, 0);
            }
        }
    }
    // tile t = (ta <= tb) of this block: 256 doubles, [i][j] = W[16 tb + i][16 ta + j] with
    // i = lane/16 + 4v, j = lane%16 (the lower triangle, which is the one k_chol factors)
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int t = wave + 4 * q;
        if (t < NTILE) {
            double* out = gram_part + (static_cast<size_t>(bid) * NTILE + t) * 256;
#pragma unroll
            for (int v = 0; v < 4; ++v) out[((lane >> 4) + 4 * v) * 16 + (lane & 15)] = acc[q][v];
        }
    }
}

// The factor P as the caller holds it (m x ldp) in the layout of ONE column split of the
// P-pass, [row][RP] with zeros from column r on: what the orthonormalisation starts from when
// P comes from outside (the second phase of a split call: P after an exchange between ranks).
__global__ __launch_bounds__(256) void k_p_to_part(const Group grp, uint32_t RP)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const uint32_t q4 = RP / 4;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x - ta.first) * 256 + threadIdx.x;
    if (i >= static_cast<uint64_t>(ta.m) * q4) return;
    const uint32_t row = static_cast<uint32_t>(i / q4), c4 = static_cast<uint32_t>(i % q4) * 4;
    const float* src = ta.P + static_cast<size_t>(row) * ta.ldp + c4;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (c4 + e < grp.r) ? src[e] : 0.0f;
    *reinterpret_cast<float4*>(ta.part + static_cast<size_t>(row) * RP + c4) = make_float4(v[0], v[1], v[2], v[3]);
}

// out[e] = sum over blocks of gp[b][e], in block order within each of four interleaved
// groups and then over the groups: a fixed tree, so the result is reproducible.
__global__ __launch_bounds__(256) void k_gram_sum(const Group grps, uint32_t ne)
{
    const TensorArgs& ta = grps.t[locate(grps, blockIdx.x)];
    const double* __restrict__ gp = ta.gram_part;
    double* __restrict__ out = ta.gram;
    const uint32_t nb = ta.d0;
    __shared__ double red[4][64];
    const uint32_t e = (blockIdx.x - ta.first) * 64 + (threadIdx.x & 63);
    const uint32_t grp = threadIdx.x >> 6;
    double s = 0.0;
    if (e < ne) {
        const double* p = gp + e;
        uint32_t b = grp;
        for (; b + 28 < nb; b += 32) {
            double x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = p[static_cast<size_t>(b + 4 * u) * ne];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += x[u];
        }
        for (; b < nb; b += 4) s += p[static_cast<size_t>(b) * ne];
    }
    red[grp][threadIdx.x & 63] = s;
    __syncthreads();
    if (grp == 0 && e < ne) out[e] = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
}

// ---------------------------------------------------------------------------
// Cholesky of the Gram matrix and the inverse factor, one block, fp64.
//   W = P^T P = L L^T,  R = L^T,  R^-1 = L^-T = X^T with X = L^-1
// Blocked right-looking factorisation on 16x16 tiles held in LDS: the diagonal
// tile is factored and inverted by one wavefront in registers (four pivots at
// a time), the panel solve, the trailing update and the blocked inverse
// X = L^-1 run on fp64 MFMA with one tile per wavefront.  X tiles below the
// diagonal are stored transposed in the (otherwise unused) upper tiles, and
// written out as tiles of R^-1 as they are finished.
// A pivot of column c not above kPivotEps W[c][c] (the scaled matrix
// D W D, D = diag(W)^-1/2, would have a pivot not above kPivotEps) marks a
// column that is numerically dependent on the previous ones: it is removed
// from the factorisation (row and column of X zero), so its P^ column is zero
// and later columns are not projected on it.
// `tiles` holds nb sets of tiles (nb > 1 only for a single tile): tile t = (ta <= tb),
// row-major over the triangle, is [i][j] = W[16 tb + i][16 ta + j].
// ---------------------------------------------------------------------------
constexpr double kPivotEps = 1e-11;
constexpr int kCholThreads = 1024;
constexpr int kCholPad = 1;      // LDS row padding of the matrix, doubles (2 and 4 measured the same or slower)

// d^-1/2 for a pivot d > 0 of the Gram matrix (a normal number: the entries are sums of squares of fp32 values): the
// hardware estimate (about 23 bits) and one third-order step y (1 + e/2 + 3 e^2 / 8), e = 1 - d y^2,
// whose error term e^3 lies below the rounding of fp64.  Four dependent operations, where the
// library routine's range handling, or two Newton steps (six), would sit on the critical path of
// the factorisation: a dependent fp64 operation costs a lone wavefront some 16 cycles.
__device__ __forceinline__ double pivot_rsq(double d)
{
    const double y = __builtin_amdgcn_rsq(d);
    const double e = fma(-(d * y), y, 1.0);
    return fma(y * e, fma(0.375, e, 0.5), y);
}

// Cholesky factorisation of a symmetric 16x16 tile and the inverse X = L^-1 of its factor, by one
// wavefront, in four block steps of four pivots.  The tile S and X (which starts as the identity)
// are held in the accumulator layout of the fp64 MFMA: register v of lane l = (j = l % 16,
// q = l / 16) holds element [q + 4v][j].  Because S stays symmetric, register b is also the MFMA
// operand of block column b: lane (i, k) holds S[i][4b + k].
// Block step b:
//   - the 4x4 diagonal block goes through LDS (`bc`, 16 doubles) to every lane, which factors it
//     in plain fp64 arithmetic, L_bb, and finds column q of X_bb = L_bb^-1 by substitution;
//   - one MFMA forms the panel in operand layout: with A = X_bb placed in rows 4b .. 4b+3 and
//     B = block column b of S, row 4b + k' of the product is L[j][k'] = sum_k X_bb[k'][k] S[j][4b+k],
//     and it lands in register b of lane (j, k');
//   - one MFMA is the rank-4 update S -= L L^T.  Rows of L above the block's end are not the
//     factor's, but an entry (i, j) of the update only takes rows i and j of L, and no entry of S
//     in those rows or columns is read again;
//   - two MFMAs apply the block row operation to X: rows of the block X_b <- X_bb X_b, then
//     rows below X_i <- X_i - L_ib X_b.  They are issued after the update of S, so that they run
//     while the next block's pivots are computed.
// A pivot of column c not above wd[c] (kPivotEps times the column's diagonal entry of the Gram matrix)
// is dead: its reciprocal root is taken as zero, so nothing is eliminated with it, and its row and
// column of X end up zero; the return value has bit c set for a dead pivot c.  `wd` and `bc` are in
// LDS.  Must be called by a whole wavefront.
__device__ __forceinline__ uint32_t chol16_factor_invert(f64x4& s, f64x4& x, int lane, double* bc, const double* wd)
{
    const int j = lane & 15, q = lane >> 4;
    uint32_t dead = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) x[v] = (q + 4 * v == j) ? 1.0 : 0.0;
    double e[4], tn[4];                                 // column q of the identity; a block's pivot thresholds
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        e[a] = (q == a) ? 1.0 : 0.0;
        tn[a] = wd[a];
    }
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int jb = j - 4 * b;
        // S[4b + a][4b + c] as it stands is register b of lane (4b + a, c)
        if (jb >= 0 && jb < 4) bc[jb * 4 + q] = s[b];
        __builtin_amdgcn_wave_barrier();
        const double a00 = bc[0], a10 = bc[4], a20 = bc[8], a30 = bc[12], a11 = bc[5], a21 = bc[9], a31 = bc[13],
                     a22 = bc[10], a32 = bc[14], a33 = bc[15];
        __builtin_amdgcn_wave_barrier();
        const double t0 = tn[0], t1 = tn[1], t2 = tn[2], t3 = tn[3];
        if (b < 3) {                                        // the next block's, off the chain
#pragma unroll
            for (int a = 0; a < 4; ++a) tn[a] = wd[4 * b + 4 + a];
        }
        const bool ok0 = a00 > t0;
        const double r0 = ok0 ? pivot_rsq(a00) : 0.0;
        const double l10 = a10 * r0, l20 = a20 * r0, l30 = a30 * r0;
        const double d1 = fma(-l10, l10, a11);
        const bool ok1 = d1 > t1;
        const double r1 = ok1 ? pivot_rsq(d1) : 0.0;
        const double l21 = fma(-l20, l10, a21) * r1, l31 = fma(-l30, l10, a31) * r1;
        const double d2 = fma(-l21, l21, fma(-l20, l20, a22));
        const bool ok2 = d2 > t2;
        const double r2 = ok2 ? pivot_rsq(d2) : 0.0;
        const double l32 = fma(-l31, l21, fma(-l30, l20, a32)) * r2;
        const double d3 = fma(-l32, l32, fma(-l31, l31, fma(-l30, l30, a33)));
        const bool ok3 = d3 > t3;
        const double r3 = ok3 ? pivot_rsq(d3) : 0.0;
        dead |= ((ok0 ? 0u : 1u) | (ok1 ? 0u : 2u) | (ok2 ? 0u : 4u) | (ok3 ? 0u : 8u)) << (4 * b);
        // column q of X_bb: L_bb x = e_q
        const double x0 = e[0] * r0;
        const double x1 = fma(-l10, x0, e[1]) * r1;
        const double x2 = fma(-l21, x1, fma(-l20, x0, e[2])) * r2;
        const double x3 = fma(-l32, x2, fma(-l31, x1, fma(-l30, x0, e[3]))) * r3;
        // lane (4b + a, k): X_bb[a][k], other lanes zero (the last pivot's entry is selected last:
        // it is the one the chain waits for)
        const double xa012 = (jb == 0) ? x0 : (jb == 1) ? x1 : (jb == 2) ? x2 : 0.0;
        const double xa = (jb == 3) ? x3 : xa012;
        const double n1 = xa - ((jb == q) ? 1.0 : 0.0);   // X_bb - I in the block's rows
        if (b < 3) {
            f64x4 lp = {0.0, 0.0, 0.0, 0.0};
            lp = __builtin_amdgcn_mfma_f64_16x16x4f64(xa, s[b], lp, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f64_16x16x4f64(-lp[b], lp[b], s, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            x = __builtin_amdgcn_mfma_f64_16x16x4f64(n1, x[b], x, 0, 0, 0);
            const double nl = (j >= 4 * b + 4) ? -lp[b] : 0.0;
            x = __builtin_amdgcn_mfma_f64_16x16x4f64(nl, x[b], x, 0, 0, 0);
        } else {
            x = __builtin_amdgcn_mfma_f64_16x16x4f64(n1, x[b], x, 0, 0, 0);
        }
    }
    return dead;
}

// Tile (i, j), i > j, of X = L^-1:  X_ij = -X_ii sum_{k=j}^{i-1} L_ik X_kj.
// A holds L in its lower tiles and X_ij transposed in the upper tile (j, i):
// A[16j + b][16i + a] = X_ij[a][b]; Xd holds the inverses of the diagonal tiles.
// chol_inverse_terms adds the terms k0 <= k < k1 of the sum to `acc`, by one wavefront; the k blocks of
// a tile alternate between two accumulators (a dependent fp64 MFMA waits some 110 cycles for the one
// before it, an independent one 64).
__device__ __forceinline__ void chol_inverse_terms(const double* A, const double* Xd, int LDA, int i, int j, int k0,
                                                   int k1, int lr, int lq, f64x4& acc)
{
    f64x4 acc2 = {0.0, 0.0, 0.0, 0.0};
    for (int k = k0; k < k1; ++k) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const double av = A[(16 * i + lr) * LDA + 16 * k + 4 * kk + lq];          // L_ik[a][kk']
            const double bv = (k == j) ? Xd[(j * 16 + 4 * kk + lq) * 17 + lr]           // X_jj[kk'][b]
                                       : A[(16 * j + lr) * LDA + 16 * k + 4 * kk + lq]; // X_kj[kk'][b]
            if (kk & 1) acc2 = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc2, 0, 0, 0);
            else acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[v] += acc2[v];
}
// The sum comes out of the MFMA in the accumulator layout, which is the layout of a B operand:
// register kk is S[4kk + lq][lr], so the product with -X_ii takes it as it stands.  The tile goes to
// LDS for the rows below and, as tile (j, i) of R^-1 = X^T, to global memory: `out` points at that
// tile ([k][c] row-major), `keep` has bit v set where entry (k = lr, c = lq + 4v) is neither beyond
// the rank nor in a removed column.
__device__ __forceinline__ void chol_inverse_store(double* A, const double* Xd, int LDA, int i, int j, int lr, int lq,
                                                   const f64x4& acc, double* __restrict__ out, uint32_t keep)
{
    f64x4 xo = {0.0, 0.0, 0.0, 0.0}, xo2 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const double av = -Xd[(i * 16 + lr) * 17 + 4 * kk + lq];                       // X_ii[a][k]
        if (kk & 1) xo2 = __builtin_amdgcn_mfma_f64_16x16x4f64(av, acc[kk], xo2, 0, 0, 0);
        else xo = __builtin_amdgcn_mfma_f64_16x16x4f64(av, acc[kk], xo, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        xo[v] += xo2[v];
        A[(16 * j + lr) * LDA + 16 * i + lq + 4 * v] = xo[v];                           // transposed
        out[lr * 16 + lq + 4 * v] = ((keep >> v) & 1u) ? xo[v] : 0.0;
    }
}

__global__ __launch_bounds__(kCholThreads) void k_chol(const Group grp, uint32_t T16)
{
    const TensorArgs& ta_ = grp.t[blockIdx.x];          // one block per tensor
    const double* __restrict__ tiles = ta_.tiles;
    double* __restrict__ rinv = ta_.rinv;
    const uint32_t nb = ta_.nb, r = grp.r;
    extern __shared__ double sm[];
    const int T = static_cast<int>(T16);
    const int RPAD = 16 * T, LDA = RPAD + kCholPad;
    double* A = sm;                                   // [RPAD][LDA]: lower tiles L, upper tiles X^T
    double* Xd = A + RPAD * LDA;                      // [T][16][17]: inverses of the diagonal tiles
    double* wd = Xd + T * 16 * 17;                    // [RPAD] kPivotEps W[c][c]: what the pivot of column c must exceed
    double* red = wd + RPAD;                          // [kCholThreads] partial sums (single tile only)
    uint32_t* deadw = reinterpret_cast<uint32_t*>(red + kCholThreads);   // [4]: bit c of the 128 set for a removed column c
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int NW = kCholThreads / 64;
    const uint32_t ntile = T16 * (T16 + 1) / 2, ne = ntile * 256;
    const int lr = lane & 15, lq = lane >> 4;         // MFMA fragment coordinates
    // ---- the Gram matrix W (lower tiles, diagonal tiles whole) into LDS ----
    // Every thread's entries are requested at once (registers).
    constexpr int kMaxPerThread = (36 * 256 + kCholThreads - 1) / kCholThreads;
    double wv[kMaxPerThread];
    f64x4 st = {0.0, 0.0, 0.0, 0.0};                  // wavefront 0: the diagonal tile of the step at hand
    if (tid < 4) deadw[tid] = 0u;
    if (nb == 1) {
#pragma unroll
        for (int u = 0; u < kMaxPerThread; ++u) {
            const uint32_t e = tid + u * kCholThreads;
            wv[u] = tiles[e < ne ? e : 0];
        }
        // wavefront 0 takes the first diagonal tile (tile 0, whole and symmetric) straight into the
        // registers it factors it from: it does not wait for the other wavefronts' entries
        if (wave == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) st[v] = tiles[(lq + 4 * v) * 16 + lr];
        }
        for (int j = tid; j < RPAD; j += kCholThreads) {
            // W[j][j] sits in diagonal tile (t, t), t = j / 16, the tile of index t T - t (t - 1) / 2
            const int t = j >> 4, ti = t * T - t * (t - 1) / 2;
            wd[j] = kPivotEps * tiles[ti * 256 + (j & 15) * 17];
        }
    }
    if (nb > 1) {                                     // ne == 256: interleaved groups of blocks per entry
        constexpr uint32_t NG = kCholThreads / 256;
        const uint32_t e = tid & 255, grp = tid >> 8;
        double sacc = 0.0;
        uint32_t b = grp;
        for (; b + 7 * NG < nb; b += 8 * NG) {
            double xx[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) xx[u] = tiles[static_cast<size_t>(b + NG * u) * ne + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) sacc += xx[u];
        }
        for (; b < nb; b += NG) sacc += tiles[static_cast<size_t>(b) * ne + e];
        red[tid] = sacc;
        __syncthreads();
        if (tid < 256) {
            double t = red[tid];
#pragma unroll
            for (uint32_t g2 = 1; g2 < NG; ++g2) t += red[tid + 256 * g2];
            red[tid] = t;
        }
        __syncthreads();
        if (tid < 16) wd[tid] = kPivotEps * red[tid * 17];
        wv[0] = red[tid & 255];
    }
    // Entry tid + u * kCholThreads sits in tile (wave / 4) + 4u, the same for a whole wavefront: the
    // tile's place (ta <= tb) is kept in scalar registers and advanced four tiles at a time.  A tile
    // holds [i][j] = W[16 tb + i][16 ta + j]: consecutive lanes write consecutive words, one LDS
    // operation per entry (the block's sixteen wavefronts share one LDS pipeline, which is what the
    // phases before and after the factorisation wait for).
    {
        int ta = 0, tb = wave >> 2;
        const int i = (tid >> 4) & 15, j = tid & 15;
#pragma unroll
        for (int u = 0; u < kMaxPerThread; ++u) {
            while (tb >= T && ta < T) { ++ta; tb = tb - T + ta; }   // row ta of the triangle has tiles tb = ta .. T-1
            if (ta < T && (nb == 1 || u == 0)) A[(16 * tb + i) * LDA + 16 * ta + j] = wv[u];
            tb += 4;
        }
    }
    if (nb > 1) {
        // a single tile summed in LDS: wavefront 0 takes it from there (its lower triangle mirrored)
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int a = lq + 4 * v, b = lr;                 // element [a][b]
                st[v] = A[max(a, b) * LDA + min(a, b)];
            }
        }
    }

    // ---- blocked right-looking Cholesky with the diagonal tile one step ahead ----
    // The serial part is the chain of diagonal tiles, so wavefront 0 does nothing else: it factors
    // tile (p, p), solves the one panel tile (p+1, p) below it, applies that tile's update to
    // (p+1, p+1) in registers and goes on to factor it.  The other wavefronts solve the rest of
    // panel p, update the rest of the trailing matrix and build X = L^-1 while wavefront 0 is on
    // the next diagonal tile.  Two block barriers per step: after X_pp and after column p of L.
    // Column j of X belongs to one wavefront, which carries the sum of a row's tile across steps:
    // the sum of row p + 1 is formed during step p (row p + 1 of L is final once panel p is, and the
    // tiles of X it takes are this wavefront's own), the product with X_(p+1)(p+1), which is all that
    // is left after the last diagonal tile, during step p + 1.  The
    // owners of the long columns sit on different SIMDs (wavefront w runs on SIMD w % 4), none on
    // wavefront 0's.
    int xcol = -1;
    {
        constexpr int owner[7] = {1, 2, 3, 7, 6, 5, 9};
#pragma unroll
        for (int j = 0; j < 7; ++j)
            if (wave == owner[j]) xcol = j;
    }
    int uslot = -1;                                      // this wavefront's place among those that update
    {
        constexpr int worker[12] = {15, 14, 13, 11, 10, 9, 5, 6, 7, 3, 2, 1};
#pragma unroll
        for (int u = 0; u < 12; ++u)
            if (wave == worker[u]) uslot = u;
    }
    f64x4 xacc = {0.0, 0.0, 0.0, 0.0};
    if (wave == 0) __builtin_amdgcn_s_setprio(3);
    for (int p = 0; p < T; ++p) {
        const int j0 = 16 * p;
        if (wave == 0) {
            f64x4 xt;
            const uint32_t dead = chol16_factor_invert(st, xt, lane, red, wd + j0);
#pragma unroll
            for (int v = 0; v < 4; ++v) Xd[(p * 16 + lq + 4 * v) * 17 + lr] = xt[v];   // X[row][col]
            if (lane == 0) deadw[p >> 1] |= dead << (16 * (p & 1));
        }
        __syncthreads();
        // panel solve: L_ip = C_ip X_pp^T, tile i = p + 1 + wave (T <= 8: one tile per wavefront at most)
        f64x4 lt = {0.0, 0.0, 0.0, 0.0};
        if (wave == 0) {
            if (p + 1 < T) {
                // wavefront 0 forms its tile transposed, L^T = X_pp C^T: register v of lane (lr, lq) is
                // L[lr][lq + 4v], which is the tile's own operand layout (k block v), so the update of
                // the next diagonal tile takes it from registers
                const int i0 = j0 + 16;
                f64x4 lt2 = {0.0, 0.0, 0.0, 0.0};               // two chains: see chol_inverse_terms
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const double av = Xd[(p * 16 + lr) * 17 + 4 * kk + lq];       // X_pp[a = lr][k]
                    const double bv = A[(i0 + lr) * LDA + j0 + 4 * kk + lq];      // C[b = lr][k]
                    if (kk & 1) lt2 = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, lt2, 0, 0, 0);
                    else lt = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, lt, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) lt[v] += lt2[v];
                // C_(p+1)(p+1) as a full symmetric tile (its lower triangle is what A holds)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int a = lq + 4 * v, b = lr;
                    st[v] = A[(i0 + max(a, b)) * LDA + i0 + min(a, b)];
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) A[(i0 + lr) * LDA + j0 + lq + 4 * v] = lt[v];
            }
        } else if (wave == NW - 1) {
            // tile (p, p) of R^-1 = X_pp^T above the diagonal: [k][c] = X_pp[c][k] for k <= c
            const uint32_t wp = deadw[p >> 1] >> (16 * (p & 1));
            double* __restrict__ out = rinv + (p * T - p * (p - 1) / 2) * 256;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const uint32_t e = lane + 64 * v, kl = e >> 4, cc = e & 15;
                const bool live = kl <= cc && 16 * p + cc < r && !((wp >> kl) & 1u) && !((wp >> cc) & 1u);
                const double xv = Xd[(p * 16 + cc) * 17 + kl];
                out[e] = live ? xv : 0.0;
            }
        } else if (p + 1 + wave < T) {
            const int i = p + 1 + wave;
            f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const double av = A[(16 * i + lr) * LDA + j0 + 4 * kk + lq];
                const double bv = Xd[(p * 16 + lr) * 17 + 4 * kk + lq];     // X_pp[b = lr][k]
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) A[(16 * i + lq + 4 * v) * LDA + j0 + lr] = acc[v];
        }
        __syncthreads();
        if (wave == 0) {
            if (p + 1 < T) {
                // the next diagonal tile: C_(p+1)(p+1) - L_(p+1)p L_(p+1)p^T, kept in registers
                f64x4 st2 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    if (kk & 1) st2 = __builtin_amdgcn_mfma_f64_16x16x4f64(-lt[kk], lt[kk], st2, 0, 0, 0);
                    else st = __builtin_amdgcn_mfma_f64_16x16x4f64(-lt[kk], lt[kk], st, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) st[v] += st2[v];
            }
        } else {
            if (xcol >= 0 && xcol < p) {
                // row p of X: the sum was formed during step p - 1; the product with -X_pp
                // entry (k, c) of R^-1 = X^T: k = 16 xcol + lr, c = 16 p + lq + 4v
                const uint32_t wk = deadw[xcol >> 1] >> (16 * (xcol & 1)), wc = deadw[p >> 1] >> (16 * (p & 1));
                uint32_t keep = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint32_t cl = lq + 4 * v;
                    if (16 * p + cl < r && !((wk >> lr) & 1u) && !((wc >> cl) & 1u)) keep |= 1u << v;
                }
                const int t = xcol * T - xcol * (xcol - 1) / 2 + (p - xcol);
                chol_inverse_store(A, Xd, LDA, p, xcol, lr, lq, xacc, rinv + t * 256, keep);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) xacc[v] = 0.0;
            if (xcol >= 0 && xcol <= p && p + 1 < T)     // row p + 1 of X: the whole sum, k = xcol .. p
                chol_inverse_terms(A, Xd, LDA, p + 1, xcol, xcol, p + 1, lr, lq, xacc);
            // trailing update: C_ic -= L_ip L_cp^T for p < c <= i, all but wavefront 0's tile (p+1, p+1),
            // by the twelve wavefronts off wavefront 0's SIMD; those that own no column of X first
            const int rem = T - p - 1, npair = rem * (rem + 1) / 2;
            for (int idx = 1 + uslot; idx < npair && uslot >= 0; idx += 12) {
                int ci, ii;                              // (c, i) offsets with c <= i, row-major over the triangle
                tri_tile(idx, rem, ci, ii);
                const int c = p + 1 + ci, i = p + 1 + ii;
                f64x4 acc;
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] = A[(16 * i + lq + 4 * v) * LDA + 16 * c + lr];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const double av = -A[(16 * i + lr) * LDA + j0 + 4 * kk + lq];
                    const double bv = A[(16 * c + lr) * LDA + j0 + 4 * kk + lq];  // L_cp[b = lr][k]
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) A[(16 * i + lq + 4 * v) * LDA + 16 * c + lr] = acc[v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// P^ = P R^-1 on fp64 MFMA (64 rows per block, 16 per wave), fp32 result in place,
// and the bf16 operand copy Pt[plane][c][i] (i contiguous, rows padded to a
// multiple of 64) that the Q-pass reads as MFMA B-fragments.
// ---------------------------------------------------------------------------
template <int T16, int NP, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void k_apply(const Group grp, uint32_t RP)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    float* __restrict__ P = ta.P;
    const double* __restrict__ rinv = ta.rinv;
    __bf16* __restrict__ pt = static_cast<__bf16*>(ta.pt);
    const uint32_t ldp = ta.ldp, m = ta.m, r = grp.r, m_pad = ta.m_pad;
    constexpr int CW = 16 * T16;
    constexpr int LD = CW + 4;             // floats; 16 rows x 4 columns per read: 2-way at worst
    constexpr int NTILE = T16 * (T16 + 1) / 2;       // upper-triangle 16x16 tiles of R^-1
    constexpr int ROWS = 16 * WAVES, NTH = 64 * WAVES;
    __shared__ __attribute__((aligned(16))) float Ps[ROWS * LD];
    __shared__ double Rs[NTILE * 256];               // tile (tk <= tc), [k][c] row-major
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t row0 = (blockIdx.x - ta.first) * ROWS;
    // R^-1 goes to LDS once per block (all loads in flight together): the multiply below then
    // runs without a round trip to L2 per k step
    // (k_chol wrote the tiles in this order, zero from rank r on)
#pragma unroll
    for (int e0 = 0; e0 < NTILE * 256; e0 += NTH) {
        const int e = e0 + tid;
        if (e < NTILE * 256) Rs[e] = rinv[e];
    }
#pragma unroll
    for (int it = 0; it < T16; ++it) {
        const int idx = tid + NTH * it;
        const int i = idx / (CW / 4), c4 = (idx % (CW / 4)) * 4;
        const uint32_t row = row0 + i;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < m) {
            const float* src = P + static_cast<size_t>(row) * ldp + c4;
            if (static_cast<uint32_t>(c4) + 4 <= r) {
                v = *reinterpret_cast<const float4*>(src);
            } else {
                if (static_cast<uint32_t>(c4) < r) v.x = src[0];
                if (static_cast<uint32_t>(c4) + 1 < r) v.y = src[1];
                if (static_cast<uint32_t>(c4) + 2 < r) v.z = src[2];
            }
        }
        *reinterpret_cast<float4*>(Ps + i * LD + c4) = v;
    }
    __syncthreads();

    f64x4 acc[T16];
#pragma unroll
    for (int tc = 0; tc < T16; ++tc) acc[tc] = f64x4{0.0, 0.0, 0.0, 0.0};
    const float* pa = Ps + (16 * wave + (lane & 15)) * LD + (lane >> 4);
    const uint32_t kq = lane >> 4, cl = lane & 15;
    const uint32_t ksteps = (r + 3) / 4;
#pragma unroll
    for (int kk = 0; kk < 4 * T16; ++kk) {
        if (static_cast<uint32_t>(kk) < ksteps) {
            const double a = static_cast<double>(pa[4 * kk]);
            const int tk = kk >> 2;
            // R^-1 is upper triangular: row tile tk only reaches column tiles tc >= tk
#pragma unroll
            for (int tc = 0; tc < T16; ++tc) {
                if (tc >= tk) {
                    const int t = tk * T16 - tk * (tk - 1) / 2 + (tc - tk);
                    const double b = Rs[t * 256 + ((kk & 3) * 4 + kq) * 16 + cl];
                    acc[tc] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[tc], 0, 0, 0);
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int tc = 0; tc < T16; ++tc)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            Ps[(16 * wave + (lane >> 4) + 4 * v) * LD + 16 * tc + (lane & 15)] = static_cast<float>(acc[tc][v]);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < T16; ++it) {
        const int idx = tid + NTH * it;
        const int i = idx / (CW / 4), c4 = (idx % (CW / 4)) * 4;
        const uint32_t row = row0 + i;
        if (row < m) {
            const float4 v = *reinterpret_cast<const float4*>(Ps + i * LD + c4);
            float* dst = P + static_cast<size_t>(row) * ldp + c4;
            if (static_cast<uint32_t>(c4) + 4 <= r) {
                *reinterpret_cast<float4*>(dst) = v;
            } else {
                if (static_cast<uint32_t>(c4) < r) dst[0] = v.x;
                if (static_cast<uint32_t>(c4) + 1 < r) dst[1] = v.y;
                if (static_cast<uint32_t>(c4) + 2 < r) dst[2] = v.z;
            }
        }
    }
    // transposed operand copy: 8 consecutive rows of one column per 16-byte store (the copy's rows are
    // padded to a multiple of 64, which a block of 128 rows may reach past)
    constexpr uint32_t SEG = ROWS / 8;
    for (uint32_t idx = tid; idx < RP * SEG; idx += NTH) {
        const uint32_t cc = idx / SEG, q = idx % SEG;
        if (row0 + 8 * q >= m_pad) continue;
        bf16x8 w[NP];
        float v8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v8[e] = (cc < static_cast<uint32_t>(CW)) ? Ps[(8 * q + e) * LD + cc] : 0.0f;
        pack8<NP>(v8, w);
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<bf16x8*>(pt + (static_cast<size_t>(p) * RP + cc) * m_pad + row0 + 8 * q) = w[p];
    }
}

// ---------------------------------------------------------------------------
// Q-pass:  Q_partial[s] = D[row-range s, :]^T * P^[row-range s, :]
// Block: 4 waves share 64-row stages; wave w owns columns [w*32*NT, (w+1)*32*NT)
// of the block's 128*NT-column strip.  Lane (jl, g) loads rows 8g..8g+7 of a
// 16-row step at columns NT*jl..NT*jl+NT-1: these are MFMA A-fragments
// (M = column, K = row) as they stand, so D is never transposed.  The P^
// operand comes from the transposed bf16 copy through a double-buffered LDS
// tile shared by the four waves (one barrier per stage).
// ---------------------------------------------------------------------------
template <int NT, bool FULL, bool STREAM>
__device__ __forceinline__ void load_d_rows(const float* __restrict__ D, uint32_t n, uint32_t m,
                                            uint32_t row_base, uint32_t col, float (&v)[8][NT])
{
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const uint32_t row = row_base + q;
        const float* p = D + static_cast<uint64_t>(row) * n + col;
        if constexpr (FULL) {
            if constexpr (NT == 4) {
                const float4 x = *reinterpret_cast<const float4*>(p);
                v[q][0] = x.x; v[q][1] = x.y; v[q][2] = x.z; v[q][3] = x.w;
            } else if constexpr (NT == 2) {
                if constexpr (STREAM) {
                    const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(p));
                    v[q][0] = x.x; v[q][1] = x.y;
                } else {
                    const float2 x = *reinterpret_cast<const float2*>(p);
                    v[q][0] = x.x; v[q][1] = x.y;
                }
            } else {
                v[q][0] = p[0];
            }
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) v[q][t] = (row < m && col + t < n) ? p[t] : 0.0f;
        }
    }
}

template <int NP, int RT, int NT, bool VECOK>
__global__ __launch_bounds__(256, (NP == 2 && RT == 4) ? 2 : 1) void k_pass_q(const Group grp)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const float* __restrict__ D = ta.E;
    const __bf16* __restrict__ pt = static_cast<const __bf16*>(ta.pt);
    float* __restrict__ part = ta.part;
    const uint32_t m_pad = ta.m_pad, m = ta.m, n = ta.n, stages_per_split = ta.d0, CB = ta.d1;
    constexpr int RP = RT * 32;
    constexpr int ROWB = NP * 128 + 16;              // LDS bytes per factor column: 64 rows x NP planes + pad
    constexpr int TILE = RP * ROWB;
    constexpr int W = 32 * NT;
    constexpr int NSEG = RP * NP * 8;                // 16-byte segments of one P^ tile
    constexpr int PS = (NSEG + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char qlds[];   // 2 tiles

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t s = lid / CB, cb = lid % CB;
    const uint32_t jw0 = cb * 4 * W + wave * W;
    const uint32_t col = jw0 + NT * jl;
    const uint32_t st_begin = s * stages_per_split;
    const uint32_t st_end = min(m_pad / 64, st_begin + stages_per_split);
    const bool cols_full = VECOK && (jw0 + W <= n);

    f32x16 acc[RT][NT];
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ct][t][v] = 0.0f;

    bf16x8 seg[PS];
    auto fetch_pt = [&](uint32_t st) {
#pragma unroll
        for (int p = 0; p < PS; ++p) {
            const int it = tid + p * 256;
            if (it < NSEG) {
                const int sg = it % 8, cp = it / 8, c = cp % RP, pl = cp / RP;
                seg[p] = *reinterpret_cast<const bf16x8*>(
                    pt + (static_cast<size_t>(pl) * RP + c) * m_pad + st * 64 + sg * 8);
            }
        }
    };
    auto store_pt = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PS; ++p) {
            const int it = tid + p * 256;
            if (it < NSEG) {
                const int sg = it % 8, cp = it / 8, c = cp % RP, pl = cp / RP;
                *reinterpret_cast<bf16x8*>(qlds + buf * TILE + c * ROWB + pl * 128 + sg * 16) = seg[p];
            }
        }
    };

    if (st_begin < st_end) fetch_pt(st_begin);
    int buf = 0;
    for (uint32_t st = st_begin; st < st_end; ++st) {
        store_pt(buf);
        __syncthreads();     // tile `buf` is complete; every wave is past its reads of stage st-2
        if (st + 1 < st_end) fetch_pt(st + 1);
        const uint32_t i0 = st * 64;
        const bool full = cols_full && (i0 + 64 <= m);
        const unsigned char* tile = qlds + buf * TILE;
        // The stage's D loads are issued at once (the other waves of the SIMD compute meanwhile);
        // fp32 above rank 64 issues them in two halves: with all 64 registers of a stage in
        // flight the kernel is 12 registers over what lets two waves share a SIMD.
        constexpr int UH = (NP == 2 && RT == 4) ? 2 : 4;
#pragma unroll
        for (int h = 0; h < 4 / UH; ++h) {
            float dv[UH][8][NT];
#pragma unroll
            for (int uu = 0; uu < UH; ++uu) {
                const int u = h * UH + uu;
                if (full) {
                    if (grp.stream) load_d_rows<NT, true, true>(D, n, m, i0 + 16 * u + 8 * g, col, dv[uu]);
                    else            load_d_rows<NT, true, false>(D, n, m, i0 + 16 * u + 8 * g, col, dv[uu]);
                } else {
                    load_d_rows<NT, false, false>(D, n, m, i0 + 16 * u + 8 * g, col, dv[uu]);
                }
            }
#pragma unroll
            for (int uu = 0; uu < UH; ++uu) {
                const int u = h * UH + uu;
                bf16x8 a[NT][NP];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    float col8[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q) col8[q] = dv[uu][q][t];
                    pack8<NP>(col8, a[t]);
                }
#pragma unroll
                for (int ct = 0; ct < RT; ++ct) {
                    bf16x8 b[NP];
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        b[p] = *reinterpret_cast<const bf16x8*>(tile + (ct * 32 + jl) * ROWB + p * 128 + u * 32 + g * 16);
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[ct][t] = mma<NP>(a[t], b, acc[ct][t]);
                }
            }
        }
        buf ^= 1;
    }

    // accumulator (ct, t, v) of lane l: column j = jw0 + NT*rho + t with rho = 8*(v/4) + 4*g + v%4,
    // factor column c = ct*32 + jl  ->  part[s][j][c]
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t j = jw0 + NT * (8 * (v / 4) + 4 * g + (v % 4)) + t;
                if (j < n) part[(static_cast<size_t>(s) * n + j) * RP + ct * 32 + jl] = acc[ct][t][v];
            }
}

// Q = sum of the row-split partials, in split order (four independent loads in flight)
__global__ __launch_bounds__(256) void k_reduce_q(const Group grp, uint32_t RP)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const float* __restrict__ part = ta.part;
    float* __restrict__ Q = ta.Q;
    const uint32_t S = ta.sq, n = ta.n, r = grp.r, ldq = ta.ldq;
    // one thread per four adjacent factor columns of one row of Q
    const uint32_t q4 = RP / 4;
    const uint64_t t = static_cast<uint64_t>(blockIdx.x - ta.first) * 256 + threadIdx.x;
    if (t >= static_cast<uint64_t>(n) * q4) return;
    const uint32_t j = static_cast<uint32_t>(t / q4), c = static_cast<uint32_t>(t % q4) * 4;
    if (c >= r) return;
    const size_t stride = static_cast<size_t>(n) * RP;
    const float* p = part + static_cast<size_t>(j) * RP + c;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    uint32_t s = 0;
    for (; s + 4 <= S; s += 4) {
        const float4 x0 = *reinterpret_cast<const float4*>(p + (s + 0) * stride);
        const float4 x1 = *reinterpret_cast<const float4*>(p + (s + 1) * stride);
        const float4 x2 = *reinterpret_cast<const float4*>(p + (s + 2) * stride);
        const float4 x3 = *reinterpret_cast<const float4*>(p + (s + 3) * stride);
        v.x += x0.x; v.y += x0.y; v.z += x0.z; v.w += x0.w;
        v.x += x1.x; v.y += x1.y; v.z += x1.z; v.w += x1.w;
        v.x += x2.x; v.y += x2.y; v.z += x2.z; v.w += x2.w;
        v.x += x3.x; v.y += x3.y; v.z += x3.z; v.w += x3.w;
    }
    for (; s < S; ++s) {
        const float4 x0 = *reinterpret_cast<const float4*>(p + s * stride);
        v.x += x0.x; v.y += x0.y; v.z += x0.z; v.w += x0.w;
    }
    float* dst = Q + static_cast<size_t>(j) * ldq + c;
    if (c + 4 <= r) {
        *reinterpret_cast<float4*>(dst) = v;              // ldq is a multiple of 4, Q 16-byte aligned
    } else {
        dst[0] = v.x;
        if (c + 1 < r) dst[1] = v.y;
        if (c + 2 < r) dst[2] = v.z;
    }
}

// ---------------------------------------------------------------------------
// Decompress:  M^ = P^ Q^T -> grad_out,  E_new = D - M^ (as transmitted), in place.
// Block: 4 waves x 32 rows; the wave's P^ rows stay in registers as A-fragments;
// Q rows of a 64-column stage go through LDS, row 2*jl + ct of the stage at LDS
// row ct*32 + jl so that every lane ends up with two adjacent columns (8-byte
// accesses, 256 B contiguous per half wave).  Q rows and D of the next stage are
// fetched while the current stage is multiplied and written.
// One bf16 plane <=> bf16 gradient and output; two planes <=> fp32.
// DEFER: only M^ is written; the residual buffer keeps D and the next step's P-pass subtracts
// M^ itself (k_pass_p_deferred).  Without DEFER a null `out` leaves the reconstruction unwritten
// (E_new alone: the deferred subtraction carried out after all).
// ---------------------------------------------------------------------------
template <int NP, int RT, bool VECOK, bool DEFER>
__global__ __launch_bounds__(256) void k_decompress(const Group grp)
{
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    const float* __restrict__ P = ta.P;
    const float* __restrict__ Q = ta.Q;
    float* __restrict__ E = ta.E;
    void* __restrict__ out_ = ta.out;
    const uint64_t ldo = ta.ldo;
    const uint32_t ldp = ta.ldp, ldq = ta.ldq, m = ta.m, n = ta.n, r = grp.r;
    const uint32_t stages_per_split = ta.d0, JS = ta.d1;
    constexpr bool OUT_BF16 = (NP == 1);
    constexpr int KT = RT * 2;                        // 16-wide k blocks over the padded rank
    constexpr int RP = RT * 32;
    constexpr int ROWB = NP * RP * 2 + 16;            // LDS bytes per Q row
    constexpr int PQ = 64 * (RP / 4) / 256;           // float4 items of the Q stage per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char dlds[];
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t js = lid % JS, rb = lid / JS;
    const uint32_t row0 = rb * 128 + wave * 32;
    const bool rows_full = row0 + 32 <= m;

    // A-fragments: row row0 + jl of P^, k = kb*16 + 8g .. +8
    bf16x8 a[KT][NP];
    {
        const uint32_t row = row0 + jl;
#pragma unroll
        for (int kb = 0; kb < KT; ++kb) {
            float v[8];
            const uint32_t c0 = kb * 16 + 8 * g;
            if (row < m && c0 + 8 <= r) {
                const float4 x = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0);
                const float4 y = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0 + 4);
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (row < m && c0 + e < r) ? P[static_cast<size_t>(row) * ldp + c0 + e] : 0.0f;
            }
            pack8<NP>(v, a[kb]);
        }
    }

    const uint32_t total_stages = (n + 63) / 64;
    const uint32_t st_begin = js * stages_per_split;
    const uint32_t st_end = min(total_stages, st_begin + stages_per_split);

    float qv[PQ][4];
    float dv[DEFER ? 1 : 2][16][2];
    auto fetch_q = [&](uint32_t st) {
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jj = idx / (RP / 4), c4 = (idx % (RP / 4)) * 4;
            const uint32_t j = st * 64 + jj;
            qv[p][0] = qv[p][1] = qv[p][2] = qv[p][3] = 0.0f;
            if (j < n && static_cast<uint32_t>(c4) < ldq) {
                const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(j) * ldq + c4);
                qv[p][0] = q.x; qv[p][1] = q.y; qv[p][2] = q.z; qv[p][3] = q.w;
            }
        }
    };
    auto stage_q = [&]() {
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jj = idx / (RP / 4), c4 = (idx % (RP / 4)) * 4;
            float m4[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) m4[e] = (static_cast<uint32_t>(c4 + e) < r) ? qv[p][e] : 0.0f;
            bf16x4 w[NP];
            pack4<NP>(m4, w);
            const int lrow = (jj & 1) * 32 + (jj >> 1);
#pragma unroll
            for (int q = 0; q < NP; ++q)
                *reinterpret_cast<bf16x4*>(dlds + lrow * ROWB + q * (RP * 2) + c4 * 2) = w[q];
        }
    };
    auto stage_full = [&](uint32_t st) { return VECOK && rows_full && st * 64 + 64 <= n; };
    // D of this lane's 16 rows x 2 adjacent columns
    auto fetch_d = [&](uint32_t st, float (&d)[16][2], auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        if constexpr (DEFER) return;
        const uint32_t col = st * 64 + 2 * jl;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = row0 + 8 * (v / 4) + 4 * g + (v % 4);
            const float* p = E + static_cast<size_t>(row) * n + col;
            if constexpr (FULL) {
                const float2 x = *reinterpret_cast<const float2*>(p);
                d[v][0] = x.x; d[v][1] = x.y;
            } else {
                d[v][0] = (row < m && col < n) ? p[0] : 0.0f;
                d[v][1] = (row < m && col + 1 < n) ? p[1] : 0.0f;
            }
        }
    };
    auto finish = [&](uint32_t st, const float (&d)[16][2], const f32x16 (&acc)[2], auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        const uint32_t col = st * 64 + 2 * jl;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = row0 + 8 * (v / 4) + 4 * g + (v % 4);
            float w0 = acc[0][v], w1 = acc[1][v];
            float* e = E + static_cast<size_t>(row) * n + col;
            if constexpr (OUT_BF16) {
                const __bf16 h0 = static_cast<__bf16>(w0), h1 = static_cast<__bf16>(w1);
                w0 = static_cast<float>(h0); w1 = static_cast<float>(h1);
                __bf16* o = static_cast<__bf16*>(out_) + static_cast<size_t>(row) * ldo + col;
                if (!DEFER && out_ == nullptr) {
                } else if constexpr (FULL) {      // the reconstruction is not read again here: past the caches
                    bf16x2 hh = {h0, h1};
                    __builtin_nontemporal_store(hh, reinterpret_cast<bf16x2*>(o));
                } else if (row < m) {
                    if (col < n) o[0] = h0;
                    if (col + 1 < n) o[1] = h1;
                }
            } else {
                float* o = static_cast<float*>(out_) + static_cast<size_t>(row) * ldo + col;
                if (!DEFER && out_ == nullptr) {
                } else if constexpr (FULL) {
                    const vf2 q2 = {w0, w1};
                    __builtin_nontemporal_store(q2, reinterpret_cast<vf2*>(o));
                } else if (row < m) {
                    if (col < n) o[0] = w0;
                    if (col + 1 < n) o[1] = w1;
                }
            }
            if constexpr (DEFER) continue;
            const float e0 = d[v][0] - w0, e1 = d[v][1] - w1;
            if constexpr (FULL) {
                *reinterpret_cast<float2*>(e) = make_float2(e0, e1);
            } else if (row < m) {
                if (col < n) e[0] = e0;
                if (col + 1 < n) e[1] = e1;
            }
        }
    };
    using T = std::true_type;
    using F = std::false_type;

    auto product = [&](f32x16 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ct][v] = 0.0f;
#pragma unroll
            for (int kb = 0; kb < KT; ++kb) {
                bf16x8 b[NP];
#pragma unroll
                for (int p = 0; p < NP; ++p)
                    b[p] = *reinterpret_cast<const bf16x8*>(dlds + (ct * 32 + jl) * ROWB + p * (RP * 2) + kb * 32 + g * 16);
                acc[ct] = mma<NP>(a[kb], b, acc[ct]);
            }
        }
    };
    auto run_stage = [&](uint32_t st, float (&dcur)[16][2], float (&dnxt)[16][2]) __attribute__((always_inline)) {
        __syncthreads();                     // previous stage's LDS reads are done
        stage_q();
        __syncthreads();
        if (st + 1 < st_end) {               // next stage's loads fly during this stage's work
            fetch_q(st + 1);
            if (stage_full(st + 1)) fetch_d(st + 1, dnxt, T{}); else fetch_d(st + 1, dnxt, F{});
        }
        f32x16 acc[2];
        product(acc);
        if (stage_full(st)) finish(st, dcur, acc, T{}); else finish(st, dcur, acc, F{});
    };
    // The same between two stages that lie wholly inside the matrix: every load is unconditional, so
    // the compiler can count them, and the wait for the Q rows at the top of a stage leaves what was
    // issued after them (the next stage's D, this stage's stores) in flight; with loads under
    // conditions it waits for everything there, the stores included.
    auto fetch_q_fast = [&](uint32_t st) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jj = idx / (RP / 4), c4 = (idx % (RP / 4)) * 4;
            // rank columns from ldq on are masked when the tile is staged: any address inside the row will do
            const uint32_t cc = min(static_cast<uint32_t>(c4), ldq - 4u);
            const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(st * 64 + jj) * ldq + cc);
            qv[p][0] = q.x; qv[p][1] = q.y; qv[p][2] = q.z; qv[p][3] = q.w;
        }
    };
    auto run_stage_fast = [&](uint32_t st, float (&dcur)[16][2], float (&dnxt)[16][2]) __attribute__((always_inline)) {
        __syncthreads();
        stage_q();
        __syncthreads();
        fetch_q_fast(st + 1);
        fetch_d(st + 1, dnxt, T{});
        f32x16 acc[2];
        product(acc);
        finish(st, dcur, acc, T{});
    };

    // stages [st_begin, fast_end) are full and followed by a full stage; they are taken in pairs
    // (the two D register sets swap roles)
    // (fp32 above rank 64: the second copy of the loop costs the two registers that let two waves
    // share a SIMD, 128 instead of 103 us on the hidden-4096 layer: left out there)
    constexpr bool FAST = !(NP == 2 && RT == 4);
    const uint32_t whole_end = (FAST && VECOK && rows_full) ? min(st_end, n / 64) : 0;
    uint32_t st = st_begin;
    if (FAST && whole_end > st_begin + 2) {
        if constexpr (FAST) {
            fetch_q_fast(st_begin);
            fetch_d(st_begin, dv[0], T{});
            for (; st + 3 <= whole_end; st += 2) {
                run_stage_fast(st, dv[0], dv[DEFER ? 0 : 1]);
                run_stage_fast(st + 1, dv[DEFER ? 0 : 1], dv[0]);
            }
        }
    } else if (st_begin < st_end) {
        fetch_q(st_begin);
        if (stage_full(st_begin)) fetch_d(st_begin, dv[0], T{}); else fetch_d(st_begin, dv[0], F{});
    }
    for (; st < st_end; st += 2) {
        run_stage(st, dv[0], dv[DEFER ? 0 : 1]);
        if (st + 1 < st_end) run_stage(st + 1, dv[DEFER ? 0 : 1], dv[0]);
    }
}

// ---------------------------------------------------------------------------
// P-pass with the deferred subtraction.  The residual buffer holds D_prev = G_prev + E_prev of
// the previous step and P, Q hold that step's factors; the residual itself is only formed here:
//   E = D_prev - M^_prev,  M^_prev = P^_prev Q_prev^T  (rounded as it was transmitted)
//   D = G + E  (written back),  P_partial[s] = D[:, k-range s] Q_prev[k-range s, :]
// so that the decompress neither reads D nor writes E: 8 bytes per element less traffic per
// step for two small MFMA products more.  M^_prev is computed exactly as k_decompress computed
// it (same fragments, same order), hence E is bit-identical to what that kernel would have
// stored.
// Block: 4 waves x 32 rows over 64-column stages, the lane layout of k_decompress (lane (jl, g)
// holds columns 2jl, 2jl+1 of 16 rows).  A stage's Q rows are staged twice: [column][rank]
// (B operand of M^) and [rank][column] (B operand of D Q); D goes through a wave-private LDS
// tile to become the A operand.
// ---------------------------------------------------------------------------
template <int NP, int RT, bool VECOK>
__global__ __launch_bounds__(256, 2) void k_pass_p_deferred(const Group grp)
{
    // Two blocks share a CU and each keeps one stage of G and D_prev in flight.  Above rank 64
    // the Q tiles of a 64-column stage would leave LDS for one block only (a version with a
    // second register set for the prefetch ran at 2.7 TB/s): k_pass_p_deferred_narrow.
    static_assert(RT <= 2, "above rank 64: k_pass_p_deferred_narrow");
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    using GT = typename GradElem<NP>::type;
    const GT* __restrict__ G = static_cast<const GT*>(ta.G);
    float* __restrict__ E = ta.E;
    const float* __restrict__ Q = ta.Q;
    const float* __restrict__ P = ta.P;
    float* __restrict__ part = ta.part;
    const uint64_t ldg = ta.ldg;
    const uint32_t ldq = ta.ldq, ldp = ta.ldp, m = ta.m, n = ta.n, r = grp.r, kper = ta.d0, S = ta.d1;
    const bool e_zero = ta.e_zero != 0;
    // without grp.defer the buffer holds E itself: the same sweep with nothing to subtract (this
    // kernel's access pattern is the faster one for bf16 gradients in either form)
    const bool subtract = grp.defer != 0 && !e_zero;
    constexpr bool ROUND_BF16 = (NP == 1);
    constexpr int KT = RT * 2, RP = RT * 32;
    constexpr int ROWQ = NP * RP * 2 + 16;            // LDS bytes per Q row, [column][rank]
    constexpr int ROWB = NP * 128 + 16;               // LDS bytes per row of 64 columns
    constexpr int PQ = 32 * (RP / 4) / 256;           // Q-stage items per thread: 2 rows x 4 ranks each
    extern __shared__ __attribute__((aligned(16))) unsigned char plds[];
    unsigned char* ldsQ = plds;                       // 64 x ROWQ
    unsigned char* ldsT = ldsQ + 64 * ROWQ;           // RP x ROWB: Q^T
    unsigned char* ldsA = ldsT + RP * ROWB;           // 128 x ROWB: D

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: row addresses then are scalar base + one per-lane offset
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t s = lid % S, rb = lid / S;
    const uint32_t row0 = rb * 128 + wave * 32;
    const uint32_t k_begin = s * kper;
    const uint32_t k_end = min(n, k_begin + kper);
    const uint32_t n_st = k_begin < k_end ? (k_end - k_begin + 63) / 64 : 0;
    const bool rows_full = row0 + 32 <= m;
    // per-lane element offsets inside a 32-row x 64-column stage (vector path: both fit 32 bits)
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
        if (subtract && row < m) {
            if (c0 + 8 <= r) {
                const float4 x = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0);
                const float4 y = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0 + 4);
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (c0 + e < r) v[e] = P[static_cast<size_t>(row) * ldp + c0 + e];
            }
        }
        pack8<NP>(v, a[kb]);
    }

    float qv[PQ][2][4];
    float dv[1][16][2], gv[1][16][2];
    auto stage_full = [&](uint32_t st) __attribute__((always_inline)) { return VECOK && rows_full && k_begin + st * 64 + 64 <= k_end; };
    // Q rows of a stage: item (jp, c4) holds rows 2jp and 2jp+1 (two adjacent columns of the
    // matrix), ranks c4 .. c4+3; lanes run along jp
    auto fetch_q = [&](uint32_t st) __attribute__((always_inline)) {
        const uint32_t col0 = k_begin + st * 64;
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jp = idx & 31, c4 = (idx >> 5) * 4;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t j = col0 + 2 * jp + h;
                qv[p][h][0] = qv[p][h][1] = qv[p][h][2] = qv[p][h][3] = 0.0f;
                if (j < n && static_cast<uint32_t>(c4) < ldq) {
                    const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(j) * ldq + c4);
                    qv[p][h][0] = q.x; qv[p][h][1] = q.y; qv[p][h][2] = q.z; qv[p][h][3] = q.w;
                }
            }
        }
    };
    // G and D_prev of this lane's 16 rows x 2 adjacent columns
    auto fetch_dg = [&](uint32_t st, auto buf_tag, auto full_tag) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_tag)::value;
        constexpr int B = decltype(buf_tag)::value;
        const uint32_t col0 = k_begin + st * 64;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t rowu = row0 + 8 * (v / 4) + (v % 4);        // scalar part of the row
            dv[B][v][0] = dv[B][v][1] = 0.0f;
            if constexpr (FULL) {
                const GT* pg = G + (static_cast<uint64_t>(rowu) * ldg + col0) + off_g;
                const float* pd = E + (static_cast<uint64_t>(rowu) * n + col0) + off_d;
                if constexpr (NP == 2) {
                    const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(pg));
                    gv[B][v][0] = x.x; gv[B][v][1] = x.y;
                } else {
                    const uint32_t x = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(pg));
                    gv[B][v][0] = __uint_as_float(x);    // the pair as loaded: widened where it is used, so
                    gv[B][v][1] = 0.0f;                  // that nothing here waits for the load
                }
                if (!e_zero) {
                    if (grp.stream) {
                        const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(pd));
                        dv[B][v][0] = x.x; dv[B][v][1] = x.y;
                    } else {
                        const float2 x = *reinterpret_cast<const float2*>(pd);
                        dv[B][v][0] = x.x; dv[B][v][1] = x.y;
                    }
                }
            } else {
                const uint32_t row = rowu + 4 * g, col = col0 + 2 * jl;
                const GT* pg = G + static_cast<uint64_t>(row) * ldg + col;
                const float* pd = E + static_cast<uint64_t>(row) * n + col;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const bool in = row < m && col + e < k_end;
                    if constexpr (NP == 2) gv[B][v][e] = in ? pg[e] : 0.0f;
                    else if (e == 0) gv[B][v][0] = __uint_as_float(in ? static_cast<uint32_t>(pg[0]) : 0u);
                    else gv[B][v][0] = __uint_as_float(__float_as_uint(gv[B][v][0]) | (in ? static_cast<uint32_t>(pg[1]) << 16 : 0u));
                    if (in && !e_zero) dv[B][v][e] = pd[e];
                }
            }
        }
    };
    // ... into LDS twice: [column][rank] (row 2jp + h at LDS row h*32 + jp, so that a lane of the
    // first product ends up with two adjacent columns) and [rank][column], there as 32-bit words
    // of two adjacent columns: 128 contiguous bytes per half wave, no 16-bit scatter
    auto stage_q = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jp = idx & 31, c4 = (idx >> 5) * 4;
            uint32_t w[2][2][NP];                      // [row h][rank pair][plane]
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float m4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) m4[e] = (static_cast<uint32_t>(c4 + e) < r) ? qv[p][h][e] : 0.0f;
                pack_pair<NP>(m4[0], m4[1], w[h][0]);
                pack_pair<NP>(m4[2], m4[3], w[h][1]);
            }
#pragma unroll
            for (int q = 0; q < NP; ++q) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const u32x2 two = {w[h][0][q], w[h][1][q]};
                    *reinterpret_cast<u32x2*>(ldsQ + (h * 32 + jp) * ROWQ + q * (RP * 2) + c4 * 2) = two;
                }
#pragma unroll
                for (int e2 = 0; e2 < 2; ++e2) {
                    // ranks c4 + 2 e2 (low halves) and c4 + 2 e2 + 1 (high halves) of the two rows
                    const uint32_t lo = __builtin_amdgcn_perm(w[1][e2][q], w[0][e2][q], 0x05040100u);
                    const uint32_t hi = __builtin_amdgcn_perm(w[1][e2][q], w[0][e2][q], 0x07060302u);
                    *reinterpret_cast<uint32_t*>(ldsT + (c4 + 2 * e2) * ROWB + q * 128 + jp * 4) = lo;
                    *reinterpret_cast<uint32_t*>(ldsT + (c4 + 2 * e2 + 1) * ROWB + q * 128 + jp * 4) = hi;
                }
            }
        }
    };

    f32x16 accp[RT];
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) accp[ct][v] = 0.0f;

    using T = std::true_type;
    using F = std::false_type;
    auto fetch_next = [&](uint32_t st, auto buf_tag) __attribute__((always_inline)) {
        if (st < n_st) { if (stage_full(st)) fetch_dg(st, buf_tag, T{}); else fetch_dg(st, buf_tag, F{}); }
    };
    using B0 = std::integral_constant<int, 0>;

    // The stage body is spelled out by macros, not lambdas: with the D / G / accumulator arrays
    // handed to a lambda the compiler spills 50 to 120 registers of the same code.
    //   M^_prev of the stage from LDS, as the decompress formed it;
    //   E = D_prev - M^_prev, D = G + E: to the residual buffer and, as bf16 planes, to the wave's LDS rows.
#define EDGC_DEFERRED_COMBINE(ST, CUR, FULL)                                                              \
    {                                                                                                     \
        const uint32_t col0 = k_begin + (ST) * 64;                                                        \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                  \
            const int rl = 8 * (v / 4) + (v % 4);                                                         \
            float w0 = acc[0][v], w1 = acc[1][v];                                                         \
            if constexpr (ROUND_BF16) {                                                                   \
                w0 = static_cast<float>(static_cast<__bf16>(w0));                                         \
                w1 = static_cast<float>(static_cast<__bf16>(w1));                                         \
            }                                                                                             \
            float g0 = gv[CUR][v][0], g1 = gv[CUR][v][1];                                                 \
            if constexpr (NP == 1) {                                                                      \
                const uint32_t bits = __float_as_uint(g0);                                                \
                g0 = __uint_as_float(bits << 16); g1 = __uint_as_float(bits & 0xffff0000u);               \
            }                                                                                             \
            const float d0 = g0 + (dv[CUR][v][0] - w0), d1 = g1 + (dv[CUR][v][1] - w1);                   \
            if constexpr (FULL) {                                                                         \
                float* pd = E + (static_cast<uint64_t>(row0 + rl) * n + col0) + off_d;                    \
                *reinterpret_cast<float2*>(pd) = make_float2(d0, d1);                                     \
            } else {                                                                                      \
                const uint32_t row = row0 + rl + 4 * g, col = col0 + 2 * jl;                              \
                float* pd = E + static_cast<uint64_t>(row) * n + col;                                     \
                if (row < m) {                                                                            \
                    if (col < k_end) pd[0] = d0;                                                          \
                    if (col + 1 < k_end) pd[1] = d1;                                                      \
                }                                                                                         \
            }                                                                                             \
            uint32_t w[NP];                                                                               \
            pack_pair<NP>(d0, d1, w);                                                                     \
            _Pragma("unroll") for (int q = 0; q < NP; ++q)                                                \
                *reinterpret_cast<uint32_t*>(ldsA + (wave * 32 + rl + 4 * g) * ROWB + q * 128 + jl * 4) = w[q]; \
        }                                                                                                 \
    }
    // One register set for G and D_prev: the next stage's loads are issued as soon as this stage
    // has used it and fly during its second product and the next stage's first one.
#define EDGC_DEFERRED_M_HAT()                                                                             \
        f32x16 acc[2];                                                                                    \
        _Pragma("unroll") for (int ct = 0; ct < 2; ++ct)                                                  \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[ct][v] = 0.0f;                             \
        if (subtract) {                                                                                   \
            _Pragma("unroll") for (int ct = 0; ct < 2; ++ct) {                                            \
                _Pragma("unroll") for (int kb = 0; kb < KT; ++kb) {                                       \
                    bf16x8 b[NP];                                                                         \
                    _Pragma("unroll") for (int p = 0; p < NP; ++p)                                        \
                        b[p] = *reinterpret_cast<const bf16x8*>(ldsQ + (ct * 32 + jl) * ROWQ + p * (RP * 2) + kb * 32 + g * 16); \
                    acc[ct] = mma<NP>(a[kb], b, acc[ct]);                                                 \
                }                                                                                         \
            }                                                                                             \
        }
#define EDGC_DEFERRED_P_PRODUCT()                                                                         \
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
        }
#define EDGC_DEFERRED_STAGE(ST, CUR, NXT)                                                                 \
    {                                                                                                     \
        __syncthreads(); /* previous stage's LDS reads are done */                                        \
        stage_q();                                                                                        \
        __syncthreads();                                                                                  \
        if ((ST) + 1 < n_st) fetch_q((ST) + 1);                                                           \
        EDGC_DEFERRED_M_HAT()                                                                             \
        if (stage_full(ST)) EDGC_DEFERRED_COMBINE(ST, CUR::value, true)                                   \
        else EDGC_DEFERRED_COMBINE(ST, CUR::value, false)                                                 \
        fetch_next((ST) + 1, NXT{});                                                                      \
        __syncthreads(); /* D tile and Q^T are in LDS */                                                  \
        EDGC_DEFERRED_P_PRODUCT()                                                                         \
    }
    // The same between two stages that lie wholly inside the matrix and the block's column range,
    // with a residual to add: every load is unconditional, so the compiler can count them and the
    // wait for the Q rows at the top of a stage leaves the G / D_prev loads behind them in flight
    // (with loads under conditions it waits for everything there).
#define EDGC_DEFERRED_STAGE_FAST(ST, STREAM)                                                              \
    {                                                                                                     \
        __syncthreads();                                                                                  \
        stage_q();                                                                                        \
        __syncthreads();                                                                                  \
        fetch_q_fast((ST) + 1);                                                                           \
        EDGC_DEFERRED_M_HAT()                                                                             \
        EDGC_DEFERRED_COMBINE(ST, 0, true)                                                                \
        fetch_dg_fast((ST) + 1, std::integral_constant<bool, STREAM>{});                                  \
        __syncthreads();                                                                                  \
        EDGC_DEFERRED_P_PRODUCT()                                                                         \
    }
    auto fetch_q_fast = [&](uint32_t st) __attribute__((always_inline)) {
        const uint32_t col0 = k_begin + st * 64;
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jp = idx & 31, c4 = (idx >> 5) * 4;
            // rank columns from ldq on are masked when the tile is staged: any address inside the row will do
            const uint32_t cc = min(static_cast<uint32_t>(c4), ldq - 4u);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(col0 + 2 * jp + h) * ldq + cc);
                qv[p][h][0] = q.x; qv[p][h][1] = q.y; qv[p][h][2] = q.z; qv[p][h][3] = q.w;
            }
        }
    };
    auto fetch_dg_fast = [&](uint32_t st, auto stream_tag) __attribute__((always_inline)) {
        constexpr bool STREAM = decltype(stream_tag)::value;
        const uint32_t col0 = k_begin + st * 64;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t rowu = row0 + 8 * (v / 4) + (v % 4);
            const GT* pg = G + (static_cast<uint64_t>(rowu) * ldg + col0) + off_g;
            const float* pd = E + (static_cast<uint64_t>(rowu) * n + col0) + off_d;
            if constexpr (NP == 2) {
                const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(pg));
                gv[0][v][0] = x.x; gv[0][v][1] = x.y;
            } else {
                gv[0][v][0] = __uint_as_float(__builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(pg)));
                gv[0][v][1] = 0.0f;
            }
            if constexpr (STREAM) {
                const vf2 x = __builtin_nontemporal_load(reinterpret_cast<const vf2*>(pd));
                dv[0][v][0] = x.x; dv[0][v][1] = x.y;
            } else {
                const float2 x = *reinterpret_cast<const float2*>(pd);
                dv[0][v][0] = x.x; dv[0][v][1] = x.y;
            }
        }
    };

    // stages [0, n_fast) are full and followed by a full stage.  (fp32 at ranks 33 to 64 has no
    // registers to spare for the second copy of the loop: it spills there and gets slower.)
    constexpr bool FAST = !(NP == 2 && RT == 2);
    const uint32_t n_whole = (FAST && VECOK && rows_full && !e_zero) ? (k_end - k_begin) / 64 : 0;
    const uint32_t n_fast = n_whole > 1 ? n_whole - 1 : 0;
    uint32_t st = 0;
    if (FAST && n_fast) {
        if constexpr (FAST) {
            fetch_q_fast(0);
            if (grp.stream) {
                fetch_dg_fast(0, T{});
                for (; st < n_fast; ++st) EDGC_DEFERRED_STAGE_FAST(st, true)
            } else {
                fetch_dg_fast(0, F{});
                for (; st < n_fast; ++st) EDGC_DEFERRED_STAGE_FAST(st, false)
            }
        }
    } else {
        if (n_st) fetch_q(0);
        fetch_next(0, B0{});
    }
    for (; st < n_st; ++st) EDGC_DEFERRED_STAGE(st, B0, B0)
#undef EDGC_DEFERRED_STAGE_FAST
#undef EDGC_DEFERRED_M_HAT
#undef EDGC_DEFERRED_P_PRODUCT
#undef EDGC_DEFERRED_STAGE
#undef EDGC_DEFERRED_COMBINE

    // partial P of this k-range: part[s][row][c], c over the padded rank
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = row0 + 8 * (v / 4) + 4 * g + (v % 4);
            if (row < m)
                part[(static_cast<size_t>(s) * m + row) * RP + ct * 32 + jl] = accp[ct][v];
        }
}

// ---------------------------------------------------------------------------
// The same pass above rank 64, where the Q tiles of a 64-column stage leave LDS for one block
// per CU only: stages of 32 columns (54 KB of LDS with fp32 gradients), so that two blocks
// share a CU again and each SIMD has two waves to overlap.  One MFMA tile per wave and stage:
// lane (jl, g) holds column jl of 16 rows, 4-byte accesses (128 contiguous bytes per half wave
// and row); neighbouring lanes swap their values (DPP) to write D into LDS as 32-bit pairs.
// Same products in the same order as k_pass_p_deferred, hence the same bits.
// ---------------------------------------------------------------------------
template <int NP, int RT, bool VECOK>
__global__ __launch_bounds__(256, 2) void k_pass_p_deferred_narrow(const Group grp)
{
    static_assert(RT == 4, "built for ranks above 64");
    const TensorArgs& ta = grp.t[locate(grp, blockIdx.x)];
    using GT = typename GradElem<NP>::type;
    const GT* __restrict__ G = static_cast<const GT*>(ta.G);
    float* __restrict__ E = ta.E;
    const float* __restrict__ Q = ta.Q;
    const float* __restrict__ P = ta.P;
    float* __restrict__ part = ta.part;
    const uint64_t ldg = ta.ldg;
    const uint32_t ldq = ta.ldq, ldp = ta.ldp, m = ta.m, n = ta.n, r = grp.r, kper = ta.d0, S = ta.d1;
    const bool e_zero = ta.e_zero != 0;
    constexpr bool ROUND_BF16 = (NP == 1);
    constexpr int KT = RT * 2, RP = RT * 32;
    constexpr int ROWQ = NP * RP * 2 + 16;            // LDS bytes per Q row, [column][rank]
    constexpr int ROWB = NP * 64 + 16;                // LDS bytes per row of 32 columns
    constexpr int PQ = 16 * (RP / 4) / 256;           // Q-stage items per thread: 2 rows x 4 ranks each
    extern __shared__ __attribute__((aligned(16))) unsigned char plds[];
    unsigned char* ldsQ = plds;                       // 32 x ROWQ
    unsigned char* ldsT = ldsQ + 32 * ROWQ;           // RP x ROWB: Q^T
    unsigned char* ldsA = ldsT + RP * ROWB;           // 128 x ROWB: D

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jl = lane & 31, g = lane >> 5;
    const uint32_t lid = blockIdx.x - ta.first;
    const uint32_t s = lid % S, rb = lid / S;
    const uint32_t row0 = rb * 128 + wave * 32;
    const uint32_t k_begin = s * kper;
    const uint32_t k_end = min(n, k_begin + kper);
    const uint32_t n_st = k_begin < k_end ? (k_end - k_begin + 31) / 32 : 0;
    const bool rows_full = row0 + 32 <= m;
    const uint32_t off_d = 4u * g * n + jl;
    const uint32_t off_g = 4u * g * static_cast<uint32_t>(ldg) + jl;

    // A-fragments of P^_prev: row row0 + jl, k = kb*16 + 8g .. +8
    bf16x8 a[KT][NP];
#pragma unroll
    for (int kb = 0; kb < KT; ++kb) {
        float v[8];
        const uint32_t row = row0 + jl, c0 = kb * 16 + 8 * g;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0.0f;
        if (!e_zero && row < m) {
            if (c0 + 8 <= r) {
                const float4 x = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0);
                const float4 y = *reinterpret_cast<const float4*>(P + static_cast<size_t>(row) * ldp + c0 + 4);
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (c0 + e < r) v[e] = P[static_cast<size_t>(row) * ldp + c0 + e];
            }
        }
        pack8<NP>(v, a[kb]);
    }

    float qv[PQ][2][4];
    float dv[16], gv[16];
    // VECOK here: n and ldg are below 2^28, so that the 32-bit lane offsets hold
    auto stage_full = [&](uint32_t st) __attribute__((always_inline)) {
        return VECOK && rows_full && k_begin + st * 32 + 32 <= k_end;
    };
    auto fetch_q = [&](uint32_t st) __attribute__((always_inline)) {
        const uint32_t col0 = k_begin + st * 32;
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jp = idx & 15, c4 = (idx >> 4) * 4;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t j = col0 + 2 * jp + h;
                qv[p][h][0] = qv[p][h][1] = qv[p][h][2] = qv[p][h][3] = 0.0f;
                if (j < n && static_cast<uint32_t>(c4) < ldq) {
                    const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(j) * ldq + c4);
                    qv[p][h][0] = q.x; qv[p][h][1] = q.y; qv[p][h][2] = q.z; qv[p][h][3] = q.w;
                }
            }
        }
    };
    auto fetch_dg = [&](uint32_t st, auto full_tag) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(full_tag)::value;
        const uint32_t col0 = k_begin + st * 32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t rowu = row0 + 8 * (v / 4) + (v % 4);
            dv[v] = 0.0f;
            if constexpr (FULL) {
                const GT* pg = G + (static_cast<uint64_t>(rowu) * ldg + col0) + off_g;
                const float* pd = E + (static_cast<uint64_t>(rowu) * n + col0) + off_d;
                if constexpr (NP == 2) gv[v] = __builtin_nontemporal_load(pg);
                else gv[v] = __uint_as_float(static_cast<uint32_t>(__builtin_nontemporal_load(pg)));   // widened where used
                if (!e_zero) dv[v] = grp.stream ? __builtin_nontemporal_load(pd) : *pd;
            } else {
                const uint32_t row = rowu + 4 * g, col = col0 + jl;
                const bool in = row < m && col < k_end;
                const GT* pg = G + static_cast<uint64_t>(row) * ldg + col;
                if constexpr (NP == 2) gv[v] = in ? *pg : 0.0f;
                else gv[v] = __uint_as_float(in ? static_cast<uint32_t>(*pg) : 0u);
                if (in && !e_zero) dv[v] = E[static_cast<uint64_t>(row) * n + col];
            }
        }
    };
    auto stage_q = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jp = idx & 15, c4 = (idx >> 4) * 4;
            uint32_t w[2][2][NP];                      // [row h][rank pair][plane]
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float m4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) m4[e] = (static_cast<uint32_t>(c4 + e) < r) ? qv[p][h][e] : 0.0f;
                pack_pair<NP>(m4[0], m4[1], w[h][0]);
                pack_pair<NP>(m4[2], m4[3], w[h][1]);
            }
#pragma unroll
            for (int q = 0; q < NP; ++q) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const u32x2 two = {w[h][0][q], w[h][1][q]};
                    *reinterpret_cast<u32x2*>(ldsQ + (2 * jp + h) * ROWQ + q * (RP * 2) + c4 * 2) = two;
                }
#pragma unroll
                for (int e2 = 0; e2 < 2; ++e2) {
                    const uint32_t lo = __builtin_amdgcn_perm(w[1][e2][q], w[0][e2][q], 0x05040100u);
                    const uint32_t hi = __builtin_amdgcn_perm(w[1][e2][q], w[0][e2][q], 0x07060302u);
                    *reinterpret_cast<uint32_t*>(ldsT + (c4 + 2 * e2) * ROWB + q * 64 + jp * 4) = lo;
                    *reinterpret_cast<uint32_t*>(ldsT + (c4 + 2 * e2 + 1) * ROWB + q * 64 + jp * 4) = hi;
                }
            }
        }
    };

    f32x16 accp[RT];
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) accp[ct][v] = 0.0f;

    using T = std::true_type;
    using F = std::false_type;
    const int odd = jl & 1;
#define EDGC_NARROW_COMBINE(ST, FULL)                                                                     \
    {                                                                                                     \
        const uint32_t col0 = k_begin + (ST) * 32;                                                        \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                  \
            const int rl = 8 * (v / 4) + (v % 4);                                                         \
            float w0 = acc[v];                                                                            \
            if constexpr (ROUND_BF16) w0 = static_cast<float>(static_cast<__bf16>(w0));                   \
            const float g0 = (NP == 1) ? __uint_as_float(__float_as_uint(gv[v]) << 16) : gv[v];           \
            const float d0 = g0 + (dv[v] - w0);                                                           \
            if constexpr (FULL) {                                                                         \
                E[(static_cast<uint64_t>(row0 + rl) * n + col0) + off_d] = d0;                            \
            } else {                                                                                      \
                const uint32_t row = row0 + rl + 4 * g, col = col0 + jl;                                  \
                if (row < m && col < k_end) E[static_cast<uint64_t>(row) * n + col] = d0;                 \
            }                                                                                             \
            /* the neighbouring column's value of the same row; even lanes write even v, odd lanes odd v */ \
            const float dn = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(d0), 0xB1, 0xF, 0xF, true)); \
            if ((v & 1) == odd) {                                                                         \
                uint32_t w[NP];                                                                           \
                pack_pair<NP>(odd ? dn : d0, odd ? d0 : dn, w);                                           \
                _Pragma("unroll") for (int q = 0; q < NP; ++q)                                            \
                    *reinterpret_cast<uint32_t*>(ldsA + (wave * 32 + rl + 4 * g) * ROWB + q * 64 + (jl >> 1) * 4) = w[q]; \
            }                                                                                             \
        }                                                                                                 \
    }

    // Stages wholly inside the matrix run through a copy of the loop whose loads are all
    // unconditional (with no residual yet, D_prev is loaded all the same and dropped), so that the
    // compiler can count what is in flight: its wait for the Q rows at the top of a stage then
    // leaves the G / D_prev loads issued behind them alone.
    auto fetch_q_fast = [&](uint32_t st) __attribute__((always_inline)) {
        const uint32_t col0 = k_begin + st * 32;
#pragma unroll
        for (int p = 0; p < PQ; ++p) {
            const int idx = tid + p * 256;
            const int jp = idx & 15, c4 = (idx >> 4) * 4;
            const uint32_t cc = min(static_cast<uint32_t>(c4), ldq - 4u);   // masked from r on when staged
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 q = *reinterpret_cast<const float4*>(Q + static_cast<size_t>(col0 + 2 * jp + h) * ldq + cc);
                qv[p][h][0] = q.x; qv[p][h][1] = q.y; qv[p][h][2] = q.z; qv[p][h][3] = q.w;
            }
        }
    };
    auto fetch_dg_fast = [&](uint32_t st, auto stream_tag) __attribute__((always_inline)) {
        constexpr bool STREAM = decltype(stream_tag)::value;
        const uint32_t col0 = k_begin + st * 32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t rowu = row0 + 8 * (v / 4) + (v % 4);
            const GT* pg = G + (static_cast<uint64_t>(rowu) * ldg + col0) + off_g;
            const float* pd = E + (static_cast<uint64_t>(rowu) * n + col0) + off_d;
            if constexpr (NP == 2) gv[v] = __builtin_nontemporal_load(pg);
            else gv[v] = __uint_as_float(static_cast<uint32_t>(__builtin_nontemporal_load(pg)));
            dv[v] = STREAM ? __builtin_nontemporal_load(pd) : *pd;
        }
    };
#define EDGC_NARROW_M_HAT()                                                                               \
        f32x16 acc;                                                                                       \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[v] = 0.0f;                                     \
        if (!e_zero) { /* M^_prev of the stage's 32 columns, as the decompress formed it */               \
            _Pragma("unroll") for (int kb = 0; kb < KT; ++kb) {                                           \
                bf16x8 b[NP];                                                                             \
                _Pragma("unroll") for (int p = 0; p < NP; ++p)                                            \
                    b[p] = *reinterpret_cast<const bf16x8*>(ldsQ + jl * ROWQ + p * (RP * 2) + kb * 32 + g * 16); \
                acc = mma<NP>(a[kb], b, acc);                                                             \
            }                                                                                             \
        }
#define EDGC_NARROW_P_PRODUCT()                                                                           \
        const unsigned char* pa = ldsA + (wave * 32 + jl) * ROWB + g * 16;                                \
        const unsigned char* pb = ldsT + jl * ROWB + g * 16;                                              \
        _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) {                                                \
            bf16x8 af[NP];                                                                                \
            _Pragma("unroll") for (int q = 0; q < NP; ++q)                                                \
                af[q] = *reinterpret_cast<const bf16x8*>(pa + q * 64 + kb * 32);                          \
            _Pragma("unroll") for (int ct = 0; ct < RT; ++ct) {                                           \
                bf16x8 b[NP];                                                                             \
                _Pragma("unroll") for (int q = 0; q < NP; ++q)                                            \
                    b[q] = *reinterpret_cast<const bf16x8*>(pb + ct * 32 * ROWB + q * 64 + kb * 32);      \
                accp[ct] = mma<NP>(af, b, accp[ct]);                                                      \
            }                                                                                             \
        }
#define EDGC_NARROW_STAGE_FAST(ST, STREAM)                                                                \
    {                                                                                                     \
        __syncthreads();                                                                                  \
        stage_q();                                                                                        \
        __syncthreads();                                                                                  \
        fetch_q_fast((ST) + 1);                                                                           \
        EDGC_NARROW_M_HAT()                                                                               \
        if (e_zero) { _Pragma("unroll") for (int v = 0; v < 16; ++v) dv[v] = 0.0f; }                      \
        EDGC_NARROW_COMBINE(ST, true)                                                                     \
        fetch_dg_fast((ST) + 1, std::integral_constant<bool, STREAM>{});                                  \
        __syncthreads();                                                                                  \
        EDGC_NARROW_P_PRODUCT()                                                                           \
    }

    // stages [0, n_fast) are full and followed by a full stage.  (With fp32 gradients the second
    // copy of the loop costs more in spilled registers than the waits it removes: bf16 only.)
    constexpr bool FAST = (NP == 1);
    const uint32_t n_whole = (FAST && VECOK && rows_full) ? (k_end - k_begin) / 32 : 0;
    const uint32_t n_fast = n_whole > 1 ? n_whole - 1 : 0;
    uint32_t st = 0;
    if (FAST && n_fast) {
        if constexpr (FAST) {
            fetch_q_fast(0);
            if (grp.stream) {
                fetch_dg_fast(0, T{});
                for (; st < n_fast; ++st) EDGC_NARROW_STAGE_FAST(st, true)
            } else {
                fetch_dg_fast(0, F{});
                for (; st < n_fast; ++st) EDGC_NARROW_STAGE_FAST(st, false)
            }
        }
    } else if (n_st) {
        fetch_q(0);
        if (stage_full(0)) fetch_dg(0, T{}); else fetch_dg(0, F{});
    }
    for (; st < n_st; ++st) {
        __syncthreads();                     // previous stage's LDS reads are done
        stage_q();
        __syncthreads();
        if (st + 1 < n_st) fetch_q(st + 1);
        EDGC_NARROW_M_HAT()
        if (stage_full(st)) EDGC_NARROW_COMBINE(st, true)
        else EDGC_NARROW_COMBINE(st, false)
        if (st + 1 < n_st) { if (stage_full(st + 1)) fetch_dg(st + 1, T{}); else fetch_dg(st + 1, F{}); }
        __syncthreads();                     // D tile and Q^T are in LDS
        EDGC_NARROW_P_PRODUCT()
    }
#undef EDGC_NARROW_STAGE_FAST
#undef EDGC_NARROW_M_HAT
#undef EDGC_NARROW_P_PRODUCT
#undef EDGC_NARROW_COMBINE

    // partial P of this k-range: part[s][row][c], c over the padded rank
#pragma unroll
    for (int ct = 0; ct < RT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t row = row0 + 8 * (v / 4) + 4 * g + (v % 4);
            if (row < m)
                part[(static_cast<size_t>(s) * m + row) * RP + ct * 32 + jl] = accp[ct][v];
        }
}

// Strided row copy (a tensor that is sent as it stands: decompress hands the gradient on).
__global__ __launch_bounds__(256) void k_copy_rows(const unsigned char* __restrict__ src, uint64_t ld_src,
                                                   unsigned char* __restrict__ dst, uint64_t ld_dst,
                                                   uint32_t m, uint64_t row_bytes)
{
    const uint64_t total = static_cast<uint64_t>(m) * row_bytes;
    for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x; i < total;
         i += static_cast<uint64_t>(gridDim.x) * 256) {
        const uint64_t row = i / row_bytes, b = i % row_bytes;
        dst[row * ld_dst + b] = src[row * ld_src + b];
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
static inline uint32_t cdiv(uint64_t a, uint64_t b) { return static_cast<uint32_t>((a + b - 1) / b); }
static inline int rank_tiles(uint32_t r) { return r <= 32 ? 1 : (r <= 64 ? 2 : 4); }

// Split-K partials: the P-pass writes at most (target blocks) * 128 rows, the
// Q-pass at most (target blocks) * 128 columns, each of the padded rank.
size_t compress_part_elems(uint64_t max_rows, uint64_t max_cols, uint32_t max_rank, int num_cu)
{
    const uint64_t RP = static_cast<uint64_t>(rank_tiles(max_rank)) * 32;
    const uint64_t target = static_cast<uint64_t>(num_cu) * 4;
    const uint64_t p_rows = std::max<uint64_t>(max_rows, 128 * target) + max_rows;
    const uint64_t q_cols = std::max<uint64_t>(max_cols, 128 * target) + max_cols;
    return static_cast<size_t>(std::max(p_rows, q_cols) * RP);
}

// Kernels that may need more than 64 KiB of dynamic LDS get the limit raised once, at context
// creation, so that hot calls make no attribute calls.
template <int NP, int RT, int NT>
static hipError_t allow_lds_pass_q()
{
    constexpr int lds = 2 * RT * 32 * (NP * 128 + 16);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_pass_q<NP, RT, NT, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_pass_q<NP, RT, NT, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

template <int NP, int RT>
static constexpr size_t deferred_lds()
{
    return static_cast<size_t>(64) * (NP * RT * 32 * 2 + 16) + static_cast<size_t>(RT * 32 + 128) * (NP * 128 + 16);
}
template <int NP, int RT>
static hipError_t allow_lds_pass_p_deferred()
{
    constexpr int lds = static_cast<int>(deferred_lds<NP, RT>());
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_pass_p_deferred<NP, RT, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_pass_p_deferred<NP, RT, false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
}

template <int NP>
static constexpr size_t deferred_narrow_lds()
{
    return static_cast<size_t>(32) * (NP * 128 * 2 + 16) + static_cast<size_t>(128 + 128) * (NP * 64 + 16);
}

int prepare_compress_kernels(edgc_ctx* ctx)
{
    constexpr int chol_max = (128 * (128 + kCholPad) + 8 * 16 * 17 + 128 + kCholThreads) * 8 + (8 + 36) * 4;
    EDGC_HIP_TRY(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(&k_chol),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, chol_max));
    EDGC_HIP_TRY(ctx, (allow_lds_pass_q<1, 4, 2>()));
    EDGC_HIP_TRY(ctx, (allow_lds_pass_q<2, 4, 2>()));
    EDGC_HIP_TRY(ctx, (allow_lds_pass_q<2, 2, 2>()));
    EDGC_HIP_TRY(ctx, (allow_lds_pass_p_deferred<2, 2>()));
    EDGC_HIP_TRY(ctx, prepare_pass_p_full());
    EDGC_HIP_TRY(ctx, prepare_decompress_full());
    return EDGC_OK;
}

int launch_init_q(edgc_ctx* ctx, float* Q, uint32_t n, uint32_t ldq, uint32_t c0, uint32_t c1,
                  uint64_t seed, hipStream_t st)
{
    const uint64_t total = static_cast<uint64_t>(n) * (c1 - c0);
    if (total == 0) return EDGC_OK;
    EDGC_LAUNCH(ctx, st, KID_INIT_Q, 4.0 * total, 0.0,
                k_init_q<<<cdiv(total, 256), 256, 0, st>>>(Q, n, ldq, c0, c1, seed));
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

int launch_copy_rows(edgc_ctx* ctx, const void* src, uint64_t ld_src, void* dst, uint64_t ld_dst,
                     uint32_t m, uint32_t n, uint32_t elem_bytes, hipStream_t st)
{
    const uint64_t total = static_cast<uint64_t>(m) * n * elem_bytes;
    if (total == 0 || src == dst) return EDGC_OK;
    const uint32_t blocks = std::min<uint32_t>(cdiv(total, 256), static_cast<uint32_t>(ctx->num_cu) * 8);
    k_copy_rows<<<blocks, 256, 0, st>>>(static_cast<const unsigned char*>(src), ld_src * elem_bytes,
                                        static_cast<unsigned char*>(dst), ld_dst * elem_bytes, m,
                                        static_cast<uint64_t>(n) * elem_bytes);
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

// The blocks a pass aims at are shared among the tensors of a group in proportion to their
// size (at least one each).
// A group whose residual (= D) takes more than half of the 256 MB last-level cache streams it
// (measured on 400 MB groups: the Q-pass reads D at 4.7 instead of 3.7 TB/s with non-temporal
// loads); a smaller one is left cached: the decompress then finds D, and the next step's P-pass
// E_new, largely still there (bench workload: 0.262 instead of 0.283 ms per step, together with
// the non-temporal store of the reconstruction).
static uint32_t group_streams(const edgc_ctx* ctx, const Group& g)
{
    if (ctx->tune_stream >= 0) return ctx->tune_stream != 0 ? 1u : 0u;
    double bytes = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) bytes += 4.0 * g.t[i].m * g.t[i].n;
    return bytes > 128.0 * 1024 * 1024 ? 1u : 0u;
}

static void share_targets(const Group& g, uint32_t target, uint32_t (&out)[kMaxGroup])
{
    double total = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) total += static_cast<double>(g.t[i].m) * g.t[i].n;
    for (uint32_t i = 0; i < g.count; ++i) {
        const double f = static_cast<double>(g.t[i].m) * g.t[i].n / total;
        out[i] = std::max<uint32_t>(1u, static_cast<uint32_t>(f * target + 0.5));
    }
}

template <int NP, int RT>
static int run_pass_p(edgc_ctx* ctx, Group& g, const TensorScratch* cap, bool with_grad, hipStream_t st)
{
    constexpr uint32_t BK = 64, RP = RT * 32;
    using GT = typename GradElem<NP>::type;
    // measured: ~4 blocks per CU stream best (3 are resident; more splits only add partials).
    // The deferred kernel above rank 64 starts every block with 64 KB of P^ fragments: there
    // exactly the two blocks per CU that are resident (0 to 7 % faster per step than four).
    // the kernels of the deferred form: above rank 64 only for that form; up to rank 64 also for bf16
    // gradients with the residual stored (its sweep is the faster one there: 295 against 390 us on the
    // hidden-5120 block)
    // groups of whole tiles with a residual to subtract: the kernel without edge paths
    constexpr edgc_dtype DT = (NP == 1) ? EDGC_BF16 : EDGC_F32;
    // eight waves per block above rank 64 (hidden-5120 bf16 block, per launch, four / eight waves: rank 128
    // 327 / 307 us; rank 64 294 / 309 us; hidden-4096 fp32 block at rank 64 233 / 243 us)
    const bool want8 = ctx->tune_pwaves == 8 || (ctx->tune_pwaves < 0 && RT == 4);
    const uint32_t pwaves = (want8 && pass_p_full_applies(g, DT, RT, 8)) ? 8u : 4u;
    // (fp32 above rank 64, whole-tile kernel against the 32-column-stage kernel: 287 against 316 us on the hidden-4096
    // block, whose residual streams from HBM; 89 against 86 us on the hidden-2048 block, which the last-level cache
    // holds: there the general kernel stays)
    const bool fp32_wide = NP == 2 && RT == 4;
    const bool use_full = with_grad && ctx->tune_full != 0 && pass_p_full_applies(g, DT, RT, pwaves) &&
                          (!fp32_wide || g.stream || ctx->tune_full > 0);
    const bool use_narrow = with_grad && g.defer && RT == 4;
    const bool use_wide = with_grad && RT <= 2 && (g.defer || NP == 1);
    const uint32_t per_cu = (use_narrow && !use_full) ? 2u : (use_full && pwaves == 8 ? 2u : 4u);
    const uint32_t rows_per_block = use_full ? 32u * pwaves : 128u;
    const uint32_t target = static_cast<uint32_t>(ctx->num_cu) * (ctx->tune_p ? ctx->tune_p : per_cu);
    uint32_t tgt[kMaxGroup];
    share_targets(g, target, tgt);
    bool vec = true;
    uint32_t blocks = 0;
    double bytes = 0.0, flops = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        const uint32_t RB = cdiv(t.m, rows_per_block), ksteps = cdiv(t.n, BK);
        uint32_t S = std::max(1u, std::min(ksteps, tgt[i] / RB));
        const uint64_t lim = cap[i].part_elems / (static_cast<uint64_t>(t.m) * RP);
        if (lim == 0) return fail(ctx, EDGC_EINVAL, "partial-factor scratch too small for this shape");
        S = static_cast<uint32_t>(std::min<uint64_t>(S, lim));
        const uint32_t kper = cdiv(ksteps, S) * BK;
        S = cdiv(t.n, kper);
        t.d0 = kper;
        t.d1 = S;
        t.sp = S;
        t.first = blocks;
        blocks += RB * S;
        // 16-byte accesses; the kernel of the deferred form reads and writes two columns per lane
        const uint32_t w = (use_wide || use_full) ? 2u : 4u;
        if (w == 2u) vec = vec && t.ldg < (1ull << 28) && t.n < (1u << 28);   // its per-lane offsets are 32-bit
        vec = vec && (t.n % w == 0) && (t.ldg % w == 0) &&
              (reinterpret_cast<uintptr_t>(t.G) % (w * sizeof(GT)) == 0) &&
              (reinterpret_cast<uintptr_t>(t.E) % (4 * w) == 0);
        // algorithmic traffic: read G (if any) and E_old (if any), write D
        const double mn = static_cast<double>(t.m) * t.n;
        bytes += mn * ((with_grad ? sizeof(GT) : 0) + (t.e_zero ? 0 : 4) + 4);
        flops += 2.0 * mn * g.r;
    }
    if (use_full) {
        // fp32 above rank 64: with the next stage's Q rows requested late the kernel spills 6 registers, early 51
        const bool qlate = ctx->tune_full == 2 || (NP == 2 && RT == 4);
        ProfScope prof_scope_(ctx, st, KID_PASS_P_DEFERRED, bytes, 2.0 * flops);
        EDGC_HIP_TRY(ctx, launch_pass_p_full(g, DT, RT, blocks, qlate, pwaves, st));
        return EDGC_OK;
    }
    if (use_narrow || use_wide) {
        // D_prev is read where the other form reads E_old: the same bytes; two products per element
        const double fl = g.defer ? 2.0 * flops : flops;
        if constexpr (RT == 4) {
            // above rank 64: 32-column stages, 4-byte accesses (no alignment beyond the element's);
            // `vec` here: the kernel's 32-bit lane offsets hold
            constexpr size_t lds = deferred_narrow_lds<NP>();
            bool off32 = true;
            for (uint32_t i = 0; i < g.count; ++i)
                off32 = off32 && g.t[i].ldg < (1ull << 28) && g.t[i].n < (1u << 28);
            if (off32)
                EDGC_LAUNCH(ctx, st, KID_PASS_P_DEFERRED, bytes, fl, (k_pass_p_deferred_narrow<NP, RT, true><<<blocks, 256, lds, st>>>(g)));
            else
                EDGC_LAUNCH(ctx, st, KID_PASS_P_DEFERRED, bytes, fl, (k_pass_p_deferred_narrow<NP, RT, false><<<blocks, 256, lds, st>>>(g)));
        } else {
            constexpr size_t lds = deferred_lds<NP, RT>();
            if (vec)
                EDGC_LAUNCH(ctx, st, KID_PASS_P_DEFERRED, bytes, fl, (k_pass_p_deferred<NP, RT, true><<<blocks, 256, lds, st>>>(g)));
            else
                EDGC_LAUNCH(ctx, st, KID_PASS_P_DEFERRED, bytes, fl, (k_pass_p_deferred<NP, RT, false><<<blocks, 256, lds, st>>>(g)));
        }
    } else if (vec)
        EDGC_LAUNCH(ctx, st, KID_PASS_P, bytes, flops, (k_pass_p<NP, RT, true><<<blocks, 256, 0, st>>>(g)));
    else
        EDGC_LAUNCH(ctx, st, KID_PASS_P, bytes, flops, (k_pass_p<NP, RT, false><<<blocks, 256, 0, st>>>(g)));
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

// sums_only: stop after P = sum of the partials (the first phase of a split call)
template <int NP>
static int run_orthonormalise(edgc_ctx* ctx, Group& g, const TensorScratch* cap, hipStream_t st,
                              bool sums_only = false)
{
    const uint32_t r = g.r;
    const uint32_t RP = rank_tiles(r) * 32;
    const uint32_t t16 = r <= 16 ? 1 : r <= 32 ? 2 : r <= 64 ? 4 : 8;   // 16-wide tiles per side
    const uint32_t ntile = t16 * (t16 + 1) / 2, ne = ntile * 256;
    uint32_t tgt[kMaxGroup];
    share_targets(g, static_cast<uint32_t>(ctx->num_cu) * 2, tgt);

    // P = sum of the partials, per-block Gram tiles
    uint32_t blocks = 0;
    double bytes = 0.0, flops = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        const uint32_t chunks = cdiv(t.m, 64);
        const uint32_t cpb = std::max(1u, chunks / tgt[i]);
        const uint32_t NB = cdiv(chunks, cpb);
        if (static_cast<uint64_t>(NB) * ne > cap[i].gram_part_elems)
            return fail(ctx, EDGC_EINVAL, "Gram scratch too small for this shape");
        t.d0 = cpb;
        t.nb = NB;
        t.first = blocks;
        blocks += NB;
        const double mr = static_cast<double>(t.m) * r;
        bytes += 4.0 * mr * (t.sp + 1);
        flops += 2.0 * mr * r;
    }
    {
        ProfScope prof_scope_(ctx, st, KID_REDUCE_GRAM, bytes, flops);
        switch (t16) {
        case 1: k_reduce_gram<1><<<blocks, 256, 0, st>>>(g, RP); break;
        case 2: k_reduce_gram<2><<<blocks, 256, 0, st>>>(g, RP); break;
        case 4: k_reduce_gram<4><<<blocks, 256, 0, st>>>(g, RP); break;
        default: k_reduce_gram<8><<<blocks, 256, 0, st>>>(g, RP); break;
        }
    }
    EDGC_HIP_TRY(ctx, hipGetLastError());
    if (sums_only) return EDGC_OK;

    // Gram = sum of the per-block tiles; the Cholesky block only sums a single tile itself
    blocks = 0;
    bytes = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        const bool summed = t.nb > 1 && t16 > 1;
        t.d0 = t.nb;
        t.first = blocks;
        if (summed) {
            blocks += cdiv(ne, 64);
            bytes += 8.0 * ne * t.nb;
        }
        t.tiles = summed ? t.gram : t.gram_part;
    }
    if (blocks) {
        EDGC_LAUNCH(ctx, st, KID_GRAM_SUM, bytes, 0.0, k_gram_sum<<<blocks, 256, 0, st>>>(g, ne));
        EDGC_HIP_TRY(ctx, hipGetLastError());
    }
    bytes = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        if (t.tiles == t.gram) t.nb = 1;
        bytes += 8.0 * ne * t.nb + 8.0 * r * r;
    }
    const size_t rpad = 16 * t16;
    const size_t chol_lds = (rpad * (rpad + kCholPad) + t16 * 16 * 17 + rpad + kCholThreads) * sizeof(double) + (8 + 36) * sizeof(uint32_t);
    EDGC_LAUNCH(ctx, st, KID_CHOL, bytes, g.count * 2.0 * r * r * r / 3.0,
                k_chol<<<g.count, kCholThreads, chol_lds, st>>>(g, t16));
    EDGC_HIP_TRY(ctx, hipGetLastError());

    // P^ = P R^-1 and its transposed bf16 copy.  Above rank 64 the 72 KB of R^-1 tiles leave room for one
    // block per CU, and a block's time is its share of fp64 MFMA work (144 per 16 rows, on four SIMDs):
    // blocks of 64 rows while they fit in one round over the CUs, of 128 rows otherwise
    uint32_t apply_rows = 64;
    if (t16 == 8) {
        uint32_t b64 = 0;
        for (uint32_t i = 0; i < g.count; ++i) b64 += cdiv(g.t[i].m_pad, 64u);
        apply_rows = ctx->tune_apply == 4 ? 64u : ctx->tune_apply == 8 ? 128u
                   : (b64 <= static_cast<uint32_t>(ctx->num_cu) ? 64u : 128u);
    }
    blocks = 0;
    bytes = flops = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        t.first = blocks;
        blocks += cdiv(t.m_pad, apply_rows);
        const double mr = static_cast<double>(t.m) * r;
        bytes += 8.0 * mr + 2.0 * NP * RP * t.m_pad;
        flops += mr * r;
    }
    {
        ProfScope prof_scope_(ctx, st, KID_APPLY, bytes, flops);
        switch (t16) {
        case 1: k_apply<1, NP, 4><<<blocks, 256, 0, st>>>(g, RP); break;
        case 2: k_apply<2, NP, 4><<<blocks, 256, 0, st>>>(g, RP); break;
        case 4: k_apply<4, NP, 4><<<blocks, 256, 0, st>>>(g, RP); break;
        default:
            if (apply_rows == 128) k_apply<8, NP, 8><<<blocks, 512, 0, st>>>(g, RP);
            else k_apply<8, NP, 4><<<blocks, 256, 0, st>>>(g, RP);
            break;
        }
    }
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

// Strip width: 128*NT columns per block; two columns per lane (256-column strips) keep two to
// three waves per SIMD, which hides the load latency, and leave room for all accumulators at
// rank 128.
template <int NP, int RT, int NT>
static int run_pass_q(edgc_ctx* ctx, Group& g, const TensorScratch* cap, hipStream_t st)
{
    constexpr uint32_t RP = RT * 32;
    constexpr size_t lds = static_cast<size_t>(2) * RP * (NP * 128 + 16);
    constexpr edgc_dtype DT = (NP == 1) ? EDGC_BF16 : EDGC_F32;
    // whole-tile groups: the pipelined kernel (pass_q_full.hip), 4 or 8 waves of 64 columns per block
    // (measured per launch, general kernel / 4 waves / 8 waves: hidden-5120 bf16 block at rank 128: 144 / 142 /
    // 132 us, at rank 64: 128 / 134 / 124, at rank 32: 128 / 132 / -; hidden-4096 fp32 block at rank 64:
    // 96 / 86 / 90; hidden-2048 fp32 block at rank 16: 21.4 / 20.5 / -)
    uint32_t qwaves = 0;
    if (NT == 2 && ctx->tune_qfull != 0) {
        const uint32_t want = ctx->tune_qfull > 0 ? (ctx->tune_qfull == 8 ? 8u : 4u)
                                                  : (NP == 1 ? (RT >= 2 ? 8u : 0u) : 4u);
        if (want && pass_q_full_applies(g, DT, RT, want)) qwaves = want;
    }
    const uint32_t W4 = (qwaves ? qwaves : 4u) * 32 * NT;
    // launches that read a gigabyte or more (a 32-tensor stage: 16 tensors share the blocks, most of them left
    // with one row split) aim at three blocks per CU: 594 against 649 us
    uint64_t d_bytes = 0;
    for (uint32_t i = 0; i < g.count; ++i) d_bytes += 4ull * g.t[i].m * g.t[i].n;
    const uint32_t per_cu = ctx->tune_q ? ctx->tune_q : (qwaves == 8 ? 1u : (d_bytes >= (1ull << 30) ? 3u : 2u));
    const uint32_t target = static_cast<uint32_t>(ctx->num_cu) * per_cu;
    uint32_t tgt[kMaxGroup];
    share_targets(g, target, tgt);
    bool vec = true;
    uint32_t blocks = 0;
    double bytes = 0.0, flops = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        const uint32_t CB = cdiv(t.n, W4), stages = t.m_pad / 64;
        uint32_t S = std::max(1u, std::min(stages, tgt[i] / CB));
        const uint64_t lim = cap[i].part_elems / (static_cast<uint64_t>(t.n) * RP);
        if (lim == 0) return fail(ctx, EDGC_EINVAL, "partial-factor scratch too small for this shape");
        S = static_cast<uint32_t>(std::min<uint64_t>(S, lim));
        const uint32_t sps = cdiv(stages, S);
        S = cdiv(stages, sps);
        t.d0 = sps;
        t.d1 = CB;
        t.sq = S;
        t.first = blocks;
        blocks += CB * S;
        vec = vec && (t.n % NT == 0) && (reinterpret_cast<uintptr_t>(t.E) % 16 == 0);
        bytes += 4.0 * t.m * t.n;
        flops += 2.0 * t.m * t.n * g.r;
    }
    if (qwaves) {
        ProfScope prof_scope_(ctx, st, KID_PASS_Q, bytes, flops);
        EDGC_HIP_TRY(ctx, launch_pass_q_full(g, DT, RT, blocks, qwaves, st));
    } else if (vec) {
        auto kern = &k_pass_q<NP, RT, NT, true>;
        EDGC_LAUNCH(ctx, st, KID_PASS_Q, bytes, flops, kern<<<blocks, 256, lds, st>>>(g));
    } else {
        auto kern = &k_pass_q<NP, RT, NT, false>;
        EDGC_LAUNCH(ctx, st, KID_PASS_Q, bytes, flops, kern<<<blocks, 256, lds, st>>>(g));
    }
    EDGC_HIP_TRY(ctx, hipGetLastError());

    blocks = 0;
    bytes = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        t.first = blocks;
        blocks += cdiv(static_cast<uint64_t>(t.n) * (RP / 4), 256);
        bytes += 4.0 * t.n * g.r * (t.sq + 1);
    }
    EDGC_LAUNCH(ctx, st, KID_REDUCE_Q, bytes, 0.0, k_reduce_q<<<blocks, 256, 0, st>>>(g, RP));
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

// phase 0: the whole step.  1: error-feedback add, P-pass and the sum of its partials: P = D Q,
// not orthonormalised.  2: P as it stands in the caller's buffer (after an exchange between
// ranks, say) is orthonormalised, then the Q-pass.  1 followed by 2 is 0 bit for bit.
template <int NP, int RT>
static int compress_impl(edgc_ctx* ctx, Group& g, const TensorScratch* cap, uint32_t power_iters,
                         int phase, hipStream_t st)
{
    for (uint32_t i = 0; i < g.count; ++i) g.t[i].m_pad = cdiv(g.t[i].m, 64) * 64;
    g.stream = group_streams(ctx, g);
    if (phase == 1) {
        int rc = run_pass_p<NP, RT>(ctx, g, cap, true, st);
        if (rc != EDGC_OK) return rc;
        return run_orthonormalise<NP>(ctx, g, cap, st, true);
    }
    if (phase == 2) {
        constexpr uint32_t RP = RT * 32;
        uint32_t blocks = 0;
        for (uint32_t i = 0; i < g.count; ++i) {
            TensorArgs& t = g.t[i];
            if (cap[i].part_elems < static_cast<uint64_t>(t.m) * RP)
                return fail(ctx, EDGC_EINVAL, "partial-factor scratch too small for this shape");
            t.sp = 1;
            t.first = blocks;
            blocks += cdiv(static_cast<uint64_t>(t.m) * (RP / 4), 256);
        }
        k_p_to_part<<<blocks, 256, 0, st>>>(g, RP);
        EDGC_HIP_TRY(ctx, hipGetLastError());
        int rc = run_orthonormalise<NP>(ctx, g, cap, st);
        if (rc != EDGC_OK) return rc;
        return run_pass_q<NP, RT, 2>(ctx, g, cap, st);
    }
    // After the first P-pass the residual buffer holds D; later iterations re-read it
    // with a null gradient (D + 0).
    for (uint32_t it = 0; it < power_iters; ++it) {
        if (it == 1)
            for (uint32_t i = 0; i < g.count; ++i) {
                g.t[i].G = nullptr;
                g.t[i].e_zero = 0;
            }
        int rc = run_pass_p<NP, RT>(ctx, g, cap, it == 0, st);
        if (rc != EDGC_OK) return rc;
        rc = run_orthonormalise<NP>(ctx, g, cap, st);
        if (rc != EDGC_OK) return rc;
        rc = run_pass_q<NP, RT, 2>(ctx, g, cap, st);
        if (rc != EDGC_OK) return rc;
    }
    return EDGC_OK;
}

int launch_compress(edgc_ctx* ctx, Group& g, const TensorScratch* cap, edgc_dtype dt,
                    uint32_t power_iters, hipStream_t st, int phase)
{
    const int rt = rank_tiles(g.r);
#define EDGC_DISPATCH(NP_)                                                        \
    switch (rt) {                                                                 \
    case 1: return compress_impl<NP_, 1>(ctx, g, cap, power_iters, phase, st);    \
    case 2: return compress_impl<NP_, 2>(ctx, g, cap, power_iters, phase, st);    \
    default: return compress_impl<NP_, 4>(ctx, g, cap, power_iters, phase, st);   \
    }
    if (dt == EDGC_BF16) { EDGC_DISPATCH(1) }
    EDGC_DISPATCH(2)
#undef EDGC_DISPATCH
}

template <int NP, int RT>
static int decompress_impl(edgc_ctx* ctx, Group& g, hipStream_t st)
{
    constexpr uint32_t RP = RT * 32;
    constexpr size_t lds = static_cast<size_t>(64) * (NP * RP * 2 + 16);
    constexpr uint32_t esz = (NP == 1) ? 2 : 4;          // one plane <=> bf16 gradient and output
    // write-only reconstruction of whole-tile groups: the kernel without edge paths, 256 rows per block
    constexpr edgc_dtype DT = (NP == 1) ? EDGC_BF16 : EDGC_F32;
    // (up to rank 64 the general kernel already writes at the rate the store pattern allows)
    const uint32_t waves = ctx->tune_dfull == 4 ? 4u : 8u;
    // also at lower ranks when the launch writes a gigabyte or more (a 32-tensor stage of hidden-4096 fp32 layers,
    // 3.2 GB per launch: 727 to 771 us against 833 to 877 at ranks 16, 32 and 64; launches of 0.2 to 0.4 GB are 1 to
    // 7 % faster through the general kernel)
    uint64_t out_bytes = 0;
    for (uint32_t i = 0; i < g.count; ++i) out_bytes += static_cast<uint64_t>(g.t[i].m) * g.t[i].n * esz;
    const bool big = out_bytes >= (1ull << 30);
    const bool use_full = g.defer && (ctx->tune_dfull > 0 || (ctx->tune_dfull < 0 && (RT == 4 || big))) &&
                          decompress_full_applies(g, DT, waves);
    const uint32_t rows_per_block = use_full ? 32u * waves : 128u;
    // (the 3.2 GB launches of that stage: four blocks per CU aimed at 717 us, two 768 us)
    const uint32_t per_cu = ctx->tune_d ? ctx->tune_d : (use_full && waves == 8 && !big ? 2u : 4u);
    const uint32_t target = static_cast<uint32_t>(ctx->num_cu) * per_cu;
    uint32_t tgt[kMaxGroup];
    share_targets(g, target, tgt);
    bool vec = true;
    uint32_t blocks = 0;
    double bytes = 0.0, flops = 0.0;
    for (uint32_t i = 0; i < g.count; ++i) {
        TensorArgs& t = g.t[i];
        const uint32_t RB = cdiv(t.m, rows_per_block), stages = cdiv(t.n, 64);
        uint32_t JS = std::max(1u, std::min(stages, tgt[i] / RB));
        const uint32_t sps = cdiv(stages, JS);
        JS = cdiv(stages, sps);
        t.d0 = sps;
        t.d1 = JS;
        t.first = blocks;
        blocks += RB * JS;
        vec = vec && (t.n % 2 == 0) && (t.ldo % 2 == 0) && (reinterpret_cast<uintptr_t>(t.E) % 8 == 0) &&
              (reinterpret_cast<uintptr_t>(t.out) % (2 * esz) == 0);
        // algorithmic traffic: write M^ (if asked for); read D and write E_new unless deferred
        bytes += static_cast<double>(t.m) * t.n * ((g.defer ? 0 : 8) + (t.out ? esz : 0));
        flops += 2.0 * t.m * t.n * g.r;
    }
    if (use_full) {
        ProfScope prof_scope_(ctx, st, KID_DECOMPRESS, bytes, flops);
        EDGC_HIP_TRY(ctx, launch_decompress_full(g, DT, RT, blocks, waves, st));
        return EDGC_OK;
    }
    if (g.defer) {
        if (vec)
            EDGC_LAUNCH(ctx, st, KID_DECOMPRESS, bytes, flops, (k_decompress<NP, RT, true, true><<<blocks, 256, lds, st>>>(g)));
        else
            EDGC_LAUNCH(ctx, st, KID_DECOMPRESS, bytes, flops, (k_decompress<NP, RT, false, true><<<blocks, 256, lds, st>>>(g)));
    } else if (vec)
        EDGC_LAUNCH(ctx, st, KID_DECOMPRESS, bytes, flops, (k_decompress<NP, RT, true, false><<<blocks, 256, lds, st>>>(g)));
    else
        EDGC_LAUNCH(ctx, st, KID_DECOMPRESS, bytes, flops, (k_decompress<NP, RT, false, false><<<blocks, 256, lds, st>>>(g)));
    EDGC_HIP_TRY(ctx, hipGetLastError());
    return EDGC_OK;
}

int launch_decompress(edgc_ctx* ctx, Group& g, edgc_dtype dt, hipStream_t st)
{
    const int rt = rank_tiles(g.r);
#define EDGC_DISPATCH(NP_)                                              \
    switch (rt) {                                                       \
    case 1: return decompress_impl<NP_, 1>(ctx, g, st);                 \
    case 2: return decompress_impl<NP_, 2>(ctx, g, st);                 \
    default: return decompress_impl<NP_, 4>(ctx, g, st);                \
    }
    if (dt == EDGC_BF16) { EDGC_DISPATCH(1) }
    EDGC_DISPATCH(2)
#undef EDGC_DISPATCH
}

}  // namespace edgc
