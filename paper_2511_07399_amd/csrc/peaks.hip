// Two microkernels that measure what this chip sustains, for the benchmark's roofline report (not part of the
// streaming path): a loop of bf16 matrix instructions with no memory traffic, and a streaming copy.
#include "common.h"

namespace sdv2 {

namespace {

// Every wave keeps eight independent 32x32 accumulators and issues v_mfma_f32_32x32x16_bf16 on them in turn, so
// that no instruction waits for its predecessor; operands stay in registers.  One workgroup of eight waves per
// compute unit (two waves per SIMD).
constexpr int kPeakAcc = 8;
__global__ __launch_bounds__(512, 1) void peak_mfma_kernel(int iters, float* sink) {
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (bf16)(0.001f * (float)((threadIdx.x + e) & 7));
        b[e] = (bf16)(0.002f * (float)((threadIdx.x * 3 + e) & 7));
    }
    f32x16 acc[kPeakAcc];
#pragma unroll
    for (int i = 0; i < kPeakAcc; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kPeakAcc; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float v = 0.0f;
#pragma unroll
    for (int i = 0; i < kPeakAcc; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) v += acc[i][r];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = v;
}

// 16 bytes per lane, four loads in flight per thread, grid-stride.
__global__ __launch_bounds__(256) void peak_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const f32x4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        dst[i] = v0;
        dst[i + stride] = v1;
        dst[i + 2 * stride] = v2;
        dst[i + 3 * stride] = v3;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_peak_mfma(int iters, int workgroups, float* sink, hipStream_t s) {
    hipLaunchKernelGGL(peak_mfma_kernel, dim3(workgroups), dim3(512), 0, s, iters, sink);
    return hipGetLastError();
}
double peak_mfma_flops(int iters, int workgroups) {
    return (double)workgroups * 8.0 * iters * kPeakAcc * 2.0 * 32 * 32 * 16;
}

hipError_t launch_peak_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    hipLaunchKernelGGL(peak_copy_kernel, dim3(256 * 8), dim3(256), 0, s, static_cast<const f32x4*>(src),
                       static_cast<f32x4*>(dst), bytes / 16);
    return hipGetLastError();
}

}  // namespace sdv2
