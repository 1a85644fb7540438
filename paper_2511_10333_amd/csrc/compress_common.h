// Device helpers shared by the compressor's translation units: MFMA operand types, the
// conversion of fp32 values to bf16 operand planes, and the lookup of a block's tensor in a
// grouped launch.
//
// MFMA 32x32x16 operand layout (64 lanes): lane l supplies A[i = l%32][k = 8*(l/32) .. +8]
// and B[k = 8*(l/32) .. +8][j = l%32]; accumulator register v of lane l holds
// D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].
#pragma once

#include "edgc_internal.h"

namespace edgc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kLdsRow = 144;   // 128 B of operand data + 16 B pad: conflict-free 16-byte reads

__device__ __forceinline__ float bf16_bits_widen(uint32_t h) { return __uint_as_float(h << 16); }

// x -> planes: p[0] = bf16(x); with two planes p[1] = bf16(x - p[0])
template <int NP>
__device__ __forceinline__ void to_planes(float x, __bf16 (&p)[NP])
{
    p[0] = static_cast<__bf16>(x);
    if constexpr (NP == 2) p[1] = static_cast<__bf16>(x - static_cast<float>(p[0]));
}

// Two floats -> packed bf16 pairs, one 32-bit word per plane (v_cvt_pk_bf16_f32, RNE):
// w[0] = (bf16(x), bf16(y)); with two planes w[1] holds the rounded remainders.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <int NP>
__device__ __forceinline__ void pack_pair(float x, float y, uint32_t (&w)[NP])
{
    const f32x2 v = {x, y};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    w[0] = __builtin_bit_cast(uint32_t, h);
    if constexpr (NP == 2) {
        const f32x2 hf = __builtin_convertvector(h, f32x2);
        const bf16x2 l = __builtin_convertvector(v - hf, bf16x2);
        w[1] = __builtin_bit_cast(uint32_t, l);
    }
}
// eight floats -> one MFMA fragment per plane
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int NP>
__device__ __forceinline__ void pack8(const float (&v)[8], bf16x8 (&f)[NP])
{
    uint32_t w[4][NP];
#pragma unroll
    for (int i = 0; i < 4; ++i) pack_pair<NP>(v[2 * i], v[2 * i + 1], w[i]);
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const u32x4 q = {w[0][p], w[1][p], w[2][p], w[3][p]};
        f[p] = __builtin_bit_cast(bf16x8, q);
    }
}
template <int NP>
__device__ __forceinline__ void pack4(const float (&v)[4], bf16x4 (&f)[NP])
{
    uint32_t w[2][NP];
    pack_pair<NP>(v[0], v[1], w[0]);
    pack_pair<NP>(v[2], v[3], w[1]);
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const u32x2 q = {w[0][p], w[1][p]};
        f[p] = __builtin_bit_cast(bf16x4, q);
    }
}

template <int NP>
__device__ __forceinline__ f32x16 mma(const bf16x8 (&a)[NP], const bf16x8 (&b)[NP], f32x16 acc)
{
    if constexpr (NP == 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[1], acc, 0, 0, 0);
    }
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], acc, 0, 0, 0);
}

// Tensor of a grouped launch that owns block `bid` (tensors with no blocks are skipped).
// Blocks keep the order of the grid: consecutive blocks, which the dispatcher spreads
// round-robin over the 8 XCDs, walk along the rows of the matrix, so that neighbouring
// 256-byte pieces of a DRAM page are requested at about the same time (measured 5 to 20 %
// faster on small matrices than giving each XCD a contiguous range of tiles; the factor
// slices the blocks share are small enough to sit in every XCD's L2).
__device__ __forceinline__ uint32_t locate(const Group& g, uint32_t bid)
{
    uint32_t t = 0;
    for (uint32_t i = 1; i < g.count; ++i) t += (bid >= g.t[i].first) ? 1u : 0u;
    return t;
}

// element type of the gradient: one bf16 plane <=> bf16 gradients (raw bits), two planes <=> fp32
template <int NP> struct GradElem { using type = float; };
template <> struct GradElem<1> { using type = uint16_t; };

typedef float vf2 __attribute__((ext_vector_type(2)));

}  // namespace edgc
