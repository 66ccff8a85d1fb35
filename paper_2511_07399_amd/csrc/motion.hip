// Motion-aware noise scheduler (StreamDiffusionV2, Section 4.1, "Motion-aware noise scheduler"):
//   d_t    = sqrt(||v_t - v_{t-1}||^2 / (C H W))                      per latent frame,
//   dhat_t = clip(max_{i in {t-k..t}} d_i / sigma, 0, 1),
//   s_t    = lambda [s_max - (s_max - s_min) dhat_t] + (1 - lambda) s_{t-1}.
// The frame differences are one pass over the latents (HBM-bound, a few hundred KB per frame); the recurrence is a
// handful of scalar operations per frame, done on the device by one wave so that s_t is there without a round trip.
#include "common.h"

namespace sdv2 {
namespace {

// grid = (kMotionBlocks, T): partial sums of (v_t - v_{t-1})^2 in fp32, one float per workgroup.
__global__ __launch_bounds__(256) void motion_diff_kernel(MotionArgs a) {
    const int t = blockIdx.y;
    const float* cur = a.frames + (size_t)t * a.n;
    const float* prev = t == 0 ? a.prev : a.frames + (size_t)(t - 1) * a.n;
    float acc = 0.0f;
    if (prev != nullptr) {
        const long long stride = (long long)gridDim.x * 256;
        const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
        if (a.vec4) {
            const f32x4* c4 = reinterpret_cast<const f32x4*>(cur);
            const f32x4* p4 = reinterpret_cast<const f32x4*>(prev);
            for (long long i = tid; i < a.n / 4; i += stride) {
                const f32x4 d = c4[i] - p4[i];
                acc += d[0] * d[0] + d[1] * d[1] + d[2] * d[2] + d[3] * d[3];
            }
        } else {
            for (long long i = tid; i < a.n; i += stride) {
                const float d = cur[i] - prev[i];
                acc += d * d;
            }
        }
    }
    __shared__ float red[4];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) a.partial[(size_t)t * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// One wave.  For t = 0 .. T-1 in order: d_t from the partial sums (added in double, fixed butterfly), then on lane 0
// the ring of the last k + 1 values, the window maximum, the clip and the moving average.
__global__ __launch_bounds__(kWave) void motion_controller_kernel(MotionArgs a, int n_blocks) {
    const int lane = threadIdx.x;
    float s = a.state[0];
    int count = __float_as_int(a.state[1]);
    float* ring = a.state + kMotionHeaderFloats;
    const int ring_len = a.k + 1;
    for (int t = 0; t < a.T; ++t) {
        double sum = 0.0;
        for (int b = lane; b < n_blocks; b += kWave) sum += (double)a.partial[(size_t)t * n_blocks + b];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
        if (lane == 0) {
            const float d = (float)sqrt(sum / (double)a.n);
            ring[count % ring_len] = d;
            ++count;
            const int have = count < ring_len ? count : ring_len;
            float mx = 0.0f;
            for (int i = 0; i < have; ++i) mx = fmaxf(mx, ring[i]);
            const float dhat = fminf(fmaxf(mx / a.sigma, 0.0f), 1.0f);
            s = a.lambda * (a.s_max - (a.s_max - a.s_min) * dhat) + (1.0f - a.lambda) * s;
            a.d_out[t] = d;
            a.dhat_out[t] = dhat;
            a.s_out[t] = s;
        }
    }
    if (lane == 0) {
        a.state[0] = s;
        a.state[1] = __int_as_float(count);
    }
}

__global__ void motion_init_kernel(float* state, int n_floats, float s_init) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_floats) state[i] = i == 0 ? s_init : 0.0f;          // count = 0 has the bit pattern of 0.0f
}

}  // namespace

hipError_t launch_motion_init(float* state, int n_floats, float s_init, hipStream_t s) {
    hipLaunchKernelGGL(motion_init_kernel, dim3((n_floats + 255) / 256), dim3(256), 0, s, state, n_floats, s_init);
    return hipGetLastError();
}

hipError_t launch_motion_update(const MotionArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(motion_diff_kernel, dim3(kMotionBlocks, a.T), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(motion_controller_kernel, dim3(1), dim3(kWave), 0, s, a, kMotionBlocks);
    return hipGetLastError();
}

}  // namespace sdv2
