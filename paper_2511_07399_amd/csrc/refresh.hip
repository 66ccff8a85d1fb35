// Adaptive sink refresh and RoPE refresh of the rolling KV cache (StreamDiffusionV2, Section 4.1, "Adaptive sink and
// RoPE refresh"): alpha_i = cos(h_t, s_i) between one frame of the chunk just appended and every sink frame, the copy
// s_i <- h_t, and the move of all cached keys by a whole number of frames in rotary phase.  All three are single
// passes over parts of one (layer, stream) cache: bound by HBM / L2 bandwidth.
#include "common.h"

namespace sdv2 {
namespace {

constexpr int kSimBlock = 256;

// Partial sums of <h, s_i>, |h|^2, |s_i|^2 over the value rows.  V^T is [H][128][cap] with a column permutation inside
// every 16 slots, so element (head, d, token j) of a frame that starts at slot s0 sits in column vt_column(s0 + j).
// grid = (blocks over the H * 128 rows, sink frames); each block writes three floats, summed in a fixed order by the
// second kernel: the result does not depend on scheduling.
__global__ __launch_bounds__(kSimBlock) void sink_similarity_partial_kernel(SinkSimArgs a) {
    const int sink = blockIdx.y;
    const int sink0 = sink * a.P;
    const int rows = a.H * kHeadDim;
    float dot = 0.0f, hh = 0.0f, ss = 0.0f;
    // Four consecutive slots that start at a multiple of four sit in four consecutive columns (the permutation
    // moves whole groups of four), so frames that start at multiples of four are read 8 bytes at a time.
    const bool quads = (a.P % 4 == 0) && (a.src0 % 4 == 0);
    for (int row = blockIdx.x; row < rows; row += gridDim.x) {
        const bf16* v = a.vt + (size_t)row * a.cap;
        if (quads) {
            for (int q = threadIdx.x; q < a.P / 4; q += kSimBlock) {
                const bf16x4 x = *reinterpret_cast<const bf16x4*>(v + vt_column(a.src0 + 4 * q));
                const bf16x4 y = *reinterpret_cast<const bf16x4*>(v + vt_column(sink0 + 4 * q));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float xf = (float)x[e], yf = (float)y[e];
                    dot += xf * yf;
                    hh += xf * xf;
                    ss += yf * yf;
                }
            }
        } else {
            for (int j = threadIdx.x; j < a.P; j += kSimBlock) {
                const float x = (float)v[vt_column(a.src0 + j)];
                const float y = (float)v[vt_column(sink0 + j)];
                dot += x * y;
                hh += x * x;
                ss += y * y;
            }
        }
    }
    __shared__ float red[3][kSimBlock / kWave];
    dot = wave_sum(dot);
    hh = wave_sum(hh);
    ss = wave_sum(ss);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        red[0][wave] = dot;
        red[1][wave] = hh;
        red[2][wave] = ss;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        float t = 0.0f;
        for (int w = 0; w < kSimBlock / kWave; ++w) t += red[threadIdx.x][w];
        a.partial[((size_t)sink * gridDim.x + blockIdx.x) * 3 + threadIdx.x] = t;
    }
}

// alpha_i = dot / sqrt(|h|^2 |s_i|^2), 0 when a norm is 0.  One wave per sink: lane l adds the partial sums of
// workgroups l, l + 64, ... in double, then the lanes are combined by a fixed butterfly.
__global__ __launch_bounds__(kWave) void sink_similarity_final_kernel(SinkSimArgs a, int n_blocks) {
    const int sink = blockIdx.x;
    const int lane = threadIdx.x;
    double acc[3] = {0.0, 0.0, 0.0};
    for (int b = lane; b < n_blocks; b += kWave) {
        const float* p = a.partial + ((size_t)sink * n_blocks + b) * 3;
        acc[0] += (double)p[0];
        acc[1] += (double)p[1];
        acc[2] += (double)p[2];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int c = 0; c < 3; ++c) acc[c] += __shfl_xor(acc[c], off, kWave);
    if (lane == 0) a.alpha[sink] = (acc[1] > 0.0 && acc[2] > 0.0) ? (float)(acc[0] / sqrt(acc[1] * acc[2])) : 0.0f;
}

// s_i <- h_t: the P key rows, value columns and token ids of the frame at slot src0 are copied to the sink frame at
// slot dst0.  Blocks [0, k_blocks) copy key rows (256 bytes per head and token, 16 bytes per lane), the rest value
// rows of V^T (P columns each) and, in the first of them, the ids.
__global__ __launch_bounds__(256) void refresh_sink_kernel(SinkCopyArgs a, int k_blocks) {
    if ((int)blockIdx.x < k_blocks) {
        // sixteen lanes per (head, token): 16 bytes each
        const int item = blockIdx.x * 16 + (threadIdx.x >> 4);
        if (item >= a.H * a.P) return;
        const int h = item / a.P, j = item - h * a.P;
        const int c = threadIdx.x & 15;
        const bf16x8* src = reinterpret_cast<const bf16x8*>(a.k + ((size_t)h * a.cap + a.src0 + j) * kHeadDim);
        bf16x8* dst = reinterpret_cast<bf16x8*>(a.k + ((size_t)h * a.cap + a.dst0 + j) * kHeadDim);
        dst[c] = src[c];
        return;
    }
    const int row = blockIdx.x - k_blocks;                       // (head, d) row of V^T
    bf16* v = a.vt + (size_t)row * a.cap;
    for (int j = threadIdx.x; j < a.P; j += 256) v[vt_column(a.dst0 + j)] = v[vt_column(a.src0 + j)];
    if (row == 0)
        for (int j = threadIdx.x; j < a.P; j += 256) a.ids[a.dst0 + j] = a.ids[a.src0 + j];
}

// Every filled slot's key, heads x frame pairs: (x0, x1) <- (x0 c - x1 s, x0 s + x1 c) with (c, s) the cosine and
// sine of -delta * omega_j, formed in double on the host (there are only kMaxFramePairs of them).
__global__ __launch_bounds__(256) void rotate_keys_kernel(RotateKeysArgs a) {
    // one thread per (head, filled slot, group of 4 pairs = 16 bytes)
    const int groups = (a.n_pairs + 3) / 4;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)a.H * a.n_slots * groups;
    if (idx >= total) return;
    const int gq = (int)(idx % groups);
    const long long t = idx / groups;
    const int si = (int)(t % a.n_slots);
    const int h = (int)(t / a.n_slots);
    const int slot = si < a.sink_fill ? si : a.S + (si - a.sink_fill);
    bf16x8* p = reinterpret_cast<bf16x8*>(a.k + ((size_t)h * a.cap + slot) * kHeadDim) + gq;
    bf16x8 x = *p;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int j = 4 * gq + e;
        if (j < a.n_pairs) {
            const float c = a.cs[j], s = a.sn[j];
            const float x0 = (float)x[2 * e], x1 = (float)x[2 * e + 1];
            x[2 * e] = (bf16)(x0 * c - x1 * s);
            x[2 * e + 1] = (bf16)(x0 * s + x1 * c);
        }
    }
    *p = x;
}

}  // namespace

int sink_similarity_blocks(int H) {
    const int rows = H * kHeadDim;
    return rows < 1024 ? rows : 1024;
}

hipError_t launch_sink_similarity(const SinkSimArgs& a, hipStream_t s) {
    const int nb = sink_similarity_blocks(a.H);
    hipLaunchKernelGGL(sink_similarity_partial_kernel, dim3(nb, a.m), dim3(kSimBlock), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sink_similarity_final_kernel, dim3(a.m), dim3(kWave), 0, s, a, nb);
    return hipGetLastError();
}

hipError_t launch_refresh_sink(const SinkCopyArgs& a, hipStream_t s) {
    const int k_blocks = (a.H * a.P + 15) / 16;
    const int v_blocks = a.H * kHeadDim;
    hipLaunchKernelGGL(refresh_sink_kernel, dim3(k_blocks + v_blocks), dim3(256), 0, s, a, k_blocks);
    return hipGetLastError();
}

hipError_t launch_rotate_keys(const RotateKeysArgs& a, hipStream_t s) {
    if (a.n_slots == 0) return hipSuccess;
    const long long total = (long long)a.H * a.n_slots * ((a.n_pairs + 3) / 4);
    hipLaunchKernelGGL(rotate_keys_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace sdv2
