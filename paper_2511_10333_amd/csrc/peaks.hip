// Measured ceilings of the device at hand, for reading the roofline figures against: what a plain
// streaming copy, a plain streaming read, a plain streaming write and a register-resident bf16 MFMA
// loop reach.  None of this is part of the method; the kernels of the hot path (Sec. II-B, IV-B,
// IV-C) are bounded by HBM, and these numbers say how much of the published peaks a kernel with no
// other work gets on this device.
#include "edgc_internal.h"

namespace edgc {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kPeakThreads = 256;
constexpr int kReadUnroll = 16;
// launch shapes that measured best on gfx950 over a sweep of grids (1 to 256 blocks per compute unit),
// loads in flight (1 to 16 per thread) and index orders (grid-stride or one contiguous range per block)
constexpr uint32_t kCopyBlocksPerCu = 4, kReadBlocksPerCu = 6, kMfmaBlocksPerCu = 4;

// dst[i] = src[i] over n4 16-byte items, grid-stride
__global__ __launch_bounds__(kPeakThreads) void k_peak_copy(const float4* __restrict__ src,
                                                            float4* __restrict__ dst, size_t n4)
{
    const size_t span = static_cast<size_t>(gridDim.x) * kPeakThreads;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kPeakThreads + threadIdx.x; i < n4; i += span)
        dst[i] = src[i];
}

// dst[i] = a constant over n4 16-byte items, grid-stride
__global__ __launch_bounds__(kPeakThreads) void k_peak_fill(float4* __restrict__ dst, size_t n4, float value)
{
    const float4 v = make_float4(value, value, value, value);
    const size_t span = static_cast<size_t>(gridDim.x) * kPeakThreads;
    for (size_t i = static_cast<size_t>(blockIdx.x) * kPeakThreads + threadIdx.x; i < n4; i += span) dst[i] = v;
}

// reads n4 16-byte items, one contiguous range per block with kReadUnroll loads per thread in flight,
// and leaves one float per thread in sink (so the loads are not dropped)
__global__ __launch_bounds__(kPeakThreads) void k_peak_read(const float4* __restrict__ src,
                                                            float* __restrict__ sink, size_t n4)
{
    const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
    const size_t begin = static_cast<size_t>(blockIdx.x) * per;
    const size_t end = begin + per < n4 ? begin + per : n4;
    float acc = 0.f;
    size_t i = begin + threadIdx.x;
    for (; i + (kReadUnroll - 1) * kPeakThreads < end; i += kReadUnroll * kPeakThreads) {
        float4 v[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) v[u] = src[i + u * kPeakThreads];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
    }
    for (; i < end; i += kPeakThreads) {
        const float4 v = src[i];
        acc += (v.x + v.y) + (v.z + v.w);
    }
    sink[static_cast<size_t>(blockIdx.x) * kPeakThreads + threadIdx.x] = acc;
}

// iters rounds of four independent 32x32x16 bf16 MFMA chains per wave, operands in registers
__global__ __launch_bounds__(kPeakThreads) void k_peak_mfma(float* __restrict__ sink, uint32_t iters)
{
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = static_cast<__bf16>(0.001f * static_cast<float>(threadIdx.x & 63) + static_cast<float>(i));
        b[i] = static_cast<__bf16>(0.5f * static_cast<float>(i) - 1.0f);
    }
    f32x16_t acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    sink[static_cast<size_t>(blockIdx.x) * kPeakThreads + threadIdx.x] = s;
}

}  // namespace
}  // namespace edgc

extern "C" int edgc_measure_device_peaks(edgc_ctx* ctx, void* buf_a, void* buf_b, uint64_t bytes,
                                         uint32_t reps, edgc_device_peaks* out, void* hip_stream)
{
    using namespace edgc;
    if (!ctx) return EDGC_EINVAL;
    if (!buf_a || !buf_b || !out || reps == 0)
        return fail(ctx, EDGC_EINVAL, "null buffer/out or reps == 0");
    if (buf_a == buf_b) return fail(ctx, EDGC_EINVAL, "the two buffers must differ");
    if ((reinterpret_cast<uintptr_t>(buf_a) | reinterpret_cast<uintptr_t>(buf_b) | bytes) & 15u)
        return fail(ctx, EDGC_EINVAL, "buffers and bytes must be multiples of 16");
    constexpr uint32_t kMfmaIters = 4096;
    const uint32_t cus = static_cast<uint32_t>(ctx->num_cu);
    const uint32_t blocks_copy = cus * kCopyBlocksPerCu, blocks_read = cus * kReadBlocksPerCu;
    const uint32_t blocks_mfma = cus * kMfmaBlocksPerCu;                     // 4 waves per SIMD
    const uint64_t sink_bytes = static_cast<uint64_t>(cus) * 8u * kPeakThreads * sizeof(float);
    static_assert(kReadBlocksPerCu <= 8 && kMfmaBlocksPerCu <= 8, "the sinks must fit the documented minimum size");
    if (bytes < sink_bytes)
        return fail(ctx, EDGC_EINVAL, "buffers too small: need at least " + std::to_string(sink_bytes) + " bytes");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    EDGC_HIP_TRY(ctx, hipSetDevice(ctx->device));
    const size_t n4 = static_cast<size_t>(bytes / 16);
    const float4* a = static_cast<const float4*>(buf_a);
    float4* b4 = static_cast<float4*>(buf_b);
    float* sink = static_cast<float*>(buf_b);
    hipEvent_t ev[2] = {nullptr, nullptr};
    int rc = EDGC_OK;
    auto hip_ok = [&](hipError_t e, const char* what) {
        if (e == hipSuccess) return true;
        rc = fail(ctx, EDGC_EHIP, std::string(what) + ": " + hipGetErrorString(e));
        return false;
    };
    for (auto& e : ev)
        if (!hip_ok(hipEventCreate(&e), "hipEventCreate")) break;
    double ms[4] = {0.0, 0.0, 0.0, 0.0};
    // the fill goes first: the buffer ends up holding the copy (behind the sinks of the last two kernels)
    const int order[4] = {3, 0, 1, 2};
    for (int oi = 0; rc == EDGC_OK && oi < 4; ++oi) {
        const int which = order[oi];
        // launch 0 is untimed
        for (uint32_t rep = 0; rc == EDGC_OK && rep <= reps; ++rep) {
            if (rep == 1 && !hip_ok(hipEventRecord(ev[0], st), "hipEventRecord")) break;
            if (which == 0)
                hipLaunchKernelGGL(k_peak_copy, dim3(blocks_copy), dim3(kPeakThreads), 0, st, a, b4, n4);
            else if (which == 1)
                hipLaunchKernelGGL(k_peak_read, dim3(blocks_read), dim3(kPeakThreads), 0, st, a, sink, n4);
            else if (which == 2)
                hipLaunchKernelGGL(k_peak_mfma, dim3(blocks_mfma), dim3(kPeakThreads), 0, st, sink, kMfmaIters);
            else
                hipLaunchKernelGGL(k_peak_fill, dim3(blocks_copy), dim3(kPeakThreads), 0, st, b4, n4, 1.0f);
            hip_ok(hipGetLastError(), "launch of a peak kernel");
        }
        if (rc != EDGC_OK) break;
        if (!hip_ok(hipEventRecord(ev[1], st), "hipEventRecord")) break;
        if (!hip_ok(hipEventSynchronize(ev[1]), "hipEventSynchronize")) break;
        float t = 0.f;
        if (!hip_ok(hipEventElapsedTime(&t, ev[0], ev[1]), "hipEventElapsedTime")) break;
        ms[which] = static_cast<double>(t) / reps;
    }
    for (auto& e : ev)
        if (e) (void)hipEventDestroy(e);
    if (rc != EDGC_OK) return rc;
    const double b = static_cast<double>(bytes);
    out->copy_gbs = 2.0 * b / (ms[0] * 1e-3) * 1e-9;
    out->read_gbs = b / (ms[1] * 1e-3) * 1e-9;
    out->write_gbs = b / (ms[3] * 1e-3) * 1e-9;
    // waves x rounds x 4 chains x (32 x 32 x 16 multiply-adds = 32768 flop)
    const double flop = static_cast<double>(blocks_mfma) * (kPeakThreads / 64) * kMfmaIters * 4.0 * 32768.0;
    out->mfma_bf16_tflops = flop / (ms[2] * 1e-3) * 1e-12;
    out->bytes = bytes;
    return EDGC_OK;
}
