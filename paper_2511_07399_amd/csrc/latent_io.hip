// Between VAE latents and the blocks' hidden state: patch gathering, un-patching, the noise rate of an incoming
// chunk and the update between denoising steps.  The paper runs its causal DiT on latents in 1-4 denoising steps per
// chunk (Section 5.1), at 2 x 2 latent positions per token (Appendix B: 1 560 tokens for a 60 x 104 latent frame) and
// sets a noise rate per chunk (Section 4.1, motion-aware noise scheduler); it prints no formula for these steps, so
// the ones here are this library's readings (stated in the header).  All of them are small HBM-bound passes; the
// two projections run on the GEMM kernel.
#include "common.h"

namespace sdv2 {

namespace {

// z fp32 [B][16][F][2 gh][2 gw] -> patches bf16 [B F gh gw][64], token (f, r, c) holding z[ch][f][2r + dr][2c + dc] at
// position 4 ch + 2 dr + dc.  One thread per (token, channel): two 8-byte loads, one 8-byte store.
__global__ __launch_bounds__(256) void patchify_kernel(const float* z, bf16* patches, int B, int F, int gh, int gw) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long P = (long long)gh * gw, L = (long long)F * P;
    if (idx >= (long long)B * L * kLatentChannels) return;
    const int ch = (int)(idx % kLatentChannels);
    const long long tok = idx / kLatentChannels;
    const int b = (int)(tok / L);
    const long long i = tok - (long long)b * L;
    const int f = (int)(i / P);
    const int r = (int)((i - (long long)f * P) / gw), c = (int)((i - (long long)f * P) % gw);
    const long long Wl = 2LL * gw, Hl = 2LL * gh;
    const float* src = z + ((((long long)b * kLatentChannels + ch) * F + f) * Hl + 2 * r) * Wl + 2 * c;
    const float2 top = *reinterpret_cast<const float2*>(src);
    const float2 bot = *reinterpret_cast<const float2*>(src + Wl);
    bf16x4 o = {(bf16)top.x, (bf16)top.y, (bf16)bot.x, (bf16)bot.y};
    *reinterpret_cast<bf16x4*>(patches + tok * (4 * kLatentChannels) + 4 * ch) = o;
}

// tokens fp32 [B F gh gw][64] -> v fp32 [B][16][F][2 gh][2 gw]: the inverse placement.
__global__ __launch_bounds__(256) void unpatchify_kernel(const float* tok, float* v, int B, int F, int gh, int gw) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long P = (long long)gh * gw, L = (long long)F * P;
    if (idx >= (long long)B * L * kLatentChannels) return;
    const int ch = (int)(idx % kLatentChannels);
    const long long t = idx / kLatentChannels;
    const int b = (int)(t / L);
    const long long i = t - (long long)b * L;
    const int f = (int)(i / P);
    const int r = (int)((i - (long long)f * P) / gw), c = (int)((i - (long long)f * P) % gw);
    const long long Wl = 2LL * gw, Hl = 2LL * gh;
    const f32x4 q = *reinterpret_cast<const f32x4*>(tok + t * (4 * kLatentChannels) + 4 * ch);
    float* dst = v + ((((long long)b * kLatentChannels + ch) * F + f) * Hl + 2 * r) * Wl + 2 * c;
    *reinterpret_cast<float2*>(dst) = float2{q[0], q[1]};
    *reinterpret_cast<float2*>(dst + Wl) = float2{q[2], q[3]};
}

struct PerStream {
    float a[kMaxBatch], b[kMaxBatch];
};

// out = (1 - s) x + s eps, s per stream
__global__ __launch_bounds__(256) void noise_kernel(const float* x, const float* eps, float* out, long long n, PerStream s) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    const long long o = (long long)blockIdx.y * n + idx;
    const float r = s.a[blockIdx.y];
    out[o] = (1.0f - r) * x[o] + r * eps[o];
}

// x0 = z - sigma v;  z_next = x0 when sigma' = 0, else (1 - sigma') x0 + sigma' eps'
__global__ __launch_bounds__(256) void sampler_kernel(const float* z, const float* v, const float* eps, float* z_next, float* x0_out,
                                                      long long n, PerStream s) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    const long long o = (long long)blockIdx.y * n + idx;
    const float sigma = s.a[blockIdx.y], sn = s.b[blockIdx.y];
    const float x0 = z[o] - sigma * v[o];
    if (x0_out != nullptr) x0_out[o] = x0;
    z_next[o] = sn == 0.0f ? x0 : (1.0f - sn) * x0 + sn * eps[o];
}

}  // namespace

hipError_t launch_patchify(const float* z, bf16* patches, int B, int F, int gh, int gw, hipStream_t s) {
    const long long n = (long long)B * F * gh * gw * kLatentChannels;
    hipLaunchKernelGGL(patchify_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, z, patches, B, F, gh, gw);
    return hipGetLastError();
}

hipError_t launch_unpatchify(const float* tok, float* v, int B, int F, int gh, int gw, hipStream_t s) {
    const long long n = (long long)B * F * gh * gw * kLatentChannels;
    hipLaunchKernelGGL(unpatchify_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, tok, v, B, F, gh, gw);
    return hipGetLastError();
}

hipError_t launch_noise(const float* x, const float* eps, float* out, int B, long long n, const float* rate, hipStream_t s) {
    PerStream ps;
    for (int b = 0; b < kMaxBatch; ++b) ps.a[b] = ps.b[b] = b < B ? rate[b] : 0.0f;
    hipLaunchKernelGGL(noise_kernel, dim3((unsigned)((n + 255) / 256), B), dim3(256), 0, s, x, eps, out, n, ps);
    return hipGetLastError();
}

hipError_t launch_sampler(const float* z, const float* v, const float* eps, float* z_next, float* x0, int B, long long n,
                          const float* sigma, const float* sigma_next, hipStream_t s) {
    PerStream ps;
    for (int b = 0; b < kMaxBatch; ++b) {
        ps.a[b] = b < B ? sigma[b] : 0.0f;
        ps.b[b] = b < B ? sigma_next[b] : 0.0f;
    }
    hipLaunchKernelGGL(sampler_kernel, dim3((unsigned)((n + 255) / 256), B), dim3(256), 0, s, z, v, eps, z_next, x0, n, ps);
    return hipGetLastError();
}

}  // namespace sdv2
