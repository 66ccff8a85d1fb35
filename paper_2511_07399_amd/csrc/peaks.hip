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

// What the LDS pipeline of a compute unit takes per wave instruction that moves a kilobyte (64 lanes x 16 bytes):
// the eight waves of one workgroup issue the same instruction back to back, `iters` rounds of eight, and wave 0 writes
// the shader clocks from the first to the last into ticks[mode].  mode 0: ds_read_b128; 1: ds_write_b128; 2: direct
// global -> LDS load of 16 bytes per lane (global_load_lds_dwordx4) from a 32 KB buffer that stays in the caches.
typedef __attribute__((address_space(3))) void* lds_void_ptr_t;
template <int MODE>
__global__ __launch_bounds__(512, 1) void peak_lds_kernel(int iters, const unsigned char* src, float* sink,
                                                           unsigned long long* ticks) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[65536];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    unsigned char* base = lds + wave * 8192;
    f32x4 v = {1.0f * lane, 2.0f, 3.0f, 4.0f};
    for (int i = threadIdx.x; i < 65536 / 16; i += 512) reinterpret_cast<f32x4*>(lds)[i] = v;
    __syncthreads();
    const unsigned long long t0 = __builtin_amdgcn_s_memtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (MODE == 0) v += *reinterpret_cast<const f32x4*>(base + u * 1024 + lane * 16);
            else if (MODE == 1) *reinterpret_cast<f32x4*>(base + u * 1024 + lane * 16) = v;
            else __builtin_amdgcn_global_load_lds(src + ((wave * 8 + u) & 31) * 1024 + lane * 16, (lds_void_ptr_t)(base + u * 1024), 16, 0, 0);
        }
        asm volatile("" ::: "memory");                 // the eight of a round stay eight: no merging across rounds
        if (MODE == 2) __builtin_amdgcn_s_waitcnt(0x0F70 | 8);      // at most one round of loads in flight behind this one
    }
    __builtin_amdgcn_s_waitcnt(0x0070);                // everything has landed (vmcnt 0, lgkmcnt 0)
    __syncthreads();
    const unsigned long long t1 = __builtin_amdgcn_s_memtime();
    sink[threadIdx.x] = v[0] + v[1] + v[2] + v[3] + reinterpret_cast<const float*>(lds)[threadIdx.x];
    if (threadIdx.x == 0) ticks[MODE] = t1 - t0;
}

}  // namespace

hipError_t launch_peak_lds(int iters, const unsigned char* src, float* sink, unsigned long long* ticks, hipStream_t s) {
    hipLaunchKernelGGL(peak_lds_kernel<0>, dim3(1), dim3(512), 0, s, iters, src, sink, ticks);
    hipLaunchKernelGGL(peak_lds_kernel<1>, dim3(1), dim3(512), 0, s, iters, src, sink, ticks);
    hipLaunchKernelGGL(peak_lds_kernel<2>, dim3(1), dim3(512), 0, s, iters, src, sink, ticks);
    return hipGetLastError();
}

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
