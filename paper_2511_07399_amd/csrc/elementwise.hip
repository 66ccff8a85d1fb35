// HBM-bound kernels of the block: LayerNorm with adaLN modulation, RMSNorm, the fused
// q/k RMSNorm + 3D-RoPE + rolling-cache append, cache re-layouts and the small conditioning GEMVs.
//
// These are the "36 b L_q C" activation bytes and the "4 b L_q C" cache write of the memory model
// in Appendix B of the paper.  The paper's implementation also pays for sliding-window buffering and
// concatenation (its measured extra traffic gamma); here a chunk's keys and values are written once,
// straight into their ring slots, and nothing is ever moved.
//
// Row reductions use cross-lane shuffles inside a wavefront (RMSNorm, the q/k norm: one wavefront per row;
// LayerNorm: two wavefronts per row that exchange their partial sums through LDS); no atomics.
#include "common.h"

namespace sdv2 {

namespace {

// physical slot of token id g:  g in the sink, else ring position
__device__ __forceinline__ int slot_of(long long g, int S, int W) {
    return g < S ? (int)g : S + (int)((g - S) % W);
}

// ------------------------------------------------------------------ LayerNorm (+ modulation or affine)
// Two wavefronts per row, two rows per workgroup: a row of the small model is only 6 KB, and with one
// wavefront per row the kernel is a chain of latencies (load, two shuffle reductions, store) on a quarter of
// the chip's wave slots.  Mean and variance come from one pass over the registers, as sums of (x - x[0])
// and (x - x[0])^2 (shifting by the row's first element keeps the fp32 variance exact enough whatever the
// row's mean); the two waves of a row exchange their partial sums through LDS.
// LN_MAXV = float4 values a lane keeps in registers: C <= 512 * LN_MAXV.
// EARLY: scale and shift are fetched together with the row instead of after the reduction.  With few rows the kernel
// is a chain of latencies and theirs would come on top of the row's; with many rows it is bound by bandwidth and the
// extra registers would only cost occupancy.
template <int LN_MAXV, bool EARLY>
__global__ __launch_bounds__(256) void layernorm_kernel(LnArgs a) {
    __shared__ float part[2][2][2];                       // [row in workgroup][wave of the row][sum, sum of squares]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rw = wave >> 1;                             // row in the workgroup
    const int half = wave & 1;
    const int t = half * 64 + lane;                       // 0 .. 127 within the row
    const int row_raw = blockIdx.x * 2 + rw;
    const bool live = row_raw < a.rows;
    const int row = live ? row_raw : a.rows - 1;          // a spare half workgroup recomputes the last row, stores nothing
    const int nvec = a.C >> 2;
    const f32x4* xp = reinterpret_cast<const f32x4*>(a.x + (size_t)row * a.C);
    const float pivot = a.x[(size_t)row * a.C];
    f32x4 v[LN_MAXV];
    f32x4 sc[EARLY ? LN_MAXV : 1], sh[EARLY ? LN_MAXV : 1];
    const int stream = row / a.rows_per_stream;
    auto fetch_affine = [&](int c, f32x4& scv, f32x4& shv) {
        scv = *reinterpret_cast<const f32x4*>(a.scale_a + c);
        shv = *reinterpret_cast<const f32x4*>(a.shift_a + c);
        if (a.scale_b != nullptr) {
            scv += *reinterpret_cast<const f32x4*>(a.scale_b + (size_t)stream * a.b_stride + c);
            shv += *reinterpret_cast<const f32x4*>(a.shift_b + (size_t)stream * a.b_stride + c);
            scv += 1.0f;
        }
    };
    float sum = 0.0f, sq = 0.0f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int idx = t + 128 * i;
        if (idx < nvec) {
            v[i] = xp[idx];
            if (EARLY) fetch_affine(idx * 4, sc[i], sh[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int idx = t + 128 * i;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float d = v[i][e] - pivot;
                sum += d;
                sq += d * d;
            }
        }
    }
    sum = wave_sum(sum);
    sq = wave_sum(sq);
    if (lane == 0) {
        part[rw][half][0] = sum;
        part[rw][half][1] = sq;
    }
    __syncthreads();
    sum = part[rw][0][0] + part[rw][1][0];
    sq = part[rw][0][1] + part[rw][1][1];
    const float inv_c = 1.0f / (float)a.C;
    const float dmean = sum * inv_c;                      // mean - pivot
    const float var = fmaxf(sq * inv_c - dmean * dmean, 0.0f);
    const float rstd = rsqrtf(var + a.eps);
    const float mean = pivot + dmean;
    if (!live) return;
    bf16* op = a.out + (size_t)row * a.C;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int idx = t + 128 * i;
        if (idx < nvec) {
            if (!EARLY) fetch_affine(idx * 4, sc[0], sh[0]);
            const f32x4 scv = sc[EARLY ? i : 0], shv = sh[EARLY ? i : 0];
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)((v[i][e] - mean) * rstd * scv[e] + shv[e]);
            *reinterpret_cast<bf16x4*>(op + idx * 4) = o;
        }
    }
}

// ------------------------------------------------------------------ RMSNorm in place on bf16 rows
// One wavefront per row; the row (NV 16-byte pieces per lane) and the gains are fetched once and stay in registers.
template <int NV>
__global__ __launch_bounds__(256) void rmsnorm_inplace_kernel(bf16* x, const float* gain, int rows, int C, int ld,
                                                              float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    bf16* xp = x + (size_t)row * ld;
    const int nvec = C >> 3;
    bf16x8 v[NV];
    f32x4 g0[NV], g1[NV];
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + 64 * i;
        if (idx < nvec) {
            v[i] = *reinterpret_cast<const bf16x8*>(xp + idx * 8);
            g0[i] = *reinterpret_cast<const f32x4*>(gain + idx * 8);
            g1[i] = *reinterpret_cast<const f32x4*>(gain + idx * 8 + 4);
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (lane + 64 * i < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sq += (float)v[i][e] * (float)v[i][e];
        }
    }
    const float r = rsqrtf(wave_sum(sq) / (float)C + eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + 64 * i;
        if (idx < nvec) {
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = (bf16)((float)v[i][e] * r * g0[i][e]);
                o[e + 4] = (bf16)((float)v[i][e + 4] * r * g1[i][e]);
            }
            *reinterpret_cast<bf16x8*>(xp + idx * 8) = o;
        }
    }
}

// ------------------------------------------------------------------ q/k RMSNorm + RoPE + append, and V^T append
// Blocks [0, norm_blocks): one wave per token.  A lane reads 16 bytes (four rotation pairs) of q and of k per
// step, four heads per wave load, keeps the row in registers, reduces the sums of squares over the whole row,
// then normalises, rotates and writes q to its buffer and k to the token's ring slot.  Lane j forms the
// rotation of pair j, in double so that the angle stays exact for any stream length, and the lanes pick
// up their four by shuffle.
// Blocks [norm_blocks, ...): one (64-token tile, head) each: v goes through LDS and is written
// transposed into the V^T cache, a slot's column given by vt_column.
constexpr int SDV2_MAX_HEADS_ROPE = 64;   // C <= 8192 and 128 channels per head
constexpr int VT_TOK = 64;
constexpr int VT_LD = kHeadDim + 2;     // LDS row stride in elements: odd number of words, no bank conflicts

__global__ __launch_bounds__(256) void rope_append_kernel(RopeAppendArgs a, int norm_blocks, int tiles_per_stream) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int C = a.C;
    if ((int)blockIdx.x < norm_blocks) {
        const int row = blockIdx.x * 4 + wave;               // over B * L
        if (row >= a.B * a.L) return;
        const int b = row / a.L;
        const int i = row - b * a.L;
        const AppendStream& st = a.st[b];
        const bf16* qp = a.qkv + (size_t)row * 3 * C;
        const bf16* kp = qp + C;
        // a wave load covers four heads: lane l holds pairs 4 (l % 16) .. + 3 of head l / 16 + 4 it
        constexpr int kMaxIt = (SDV2_MAX_HEADS_ROPE + 3) / 4;
        const int hl = lane >> 4;
        const int p0 = 4 * (lane & 15);                      // first of this lane's four rotation pairs
        bf16x8 qv[kMaxIt], kv[kMaxIt];
        float sq = 0.0f, sk = 0.0f;
#pragma unroll
        for (int it = 0; it < kMaxIt; ++it) {
            const int h = hl + 4 * it;
            if (h < a.H) {
                qv[it] = *reinterpret_cast<const bf16x8*>(qp + h * kHeadDim + 2 * p0);
                kv[it] = *reinterpret_cast<const bf16x8*>(kp + h * kHeadDim + 2 * p0);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    sq += (float)qv[it][e] * (float)qv[it][e];
                    sk += (float)kv[it][e] * (float)kv[it][e];
                }
            }
        }
        const float rq = rsqrtf(wave_sum(sq) / (float)C + a.eps);
        const float rk = rsqrtf(wave_sum(sk) / (float)C + a.eps);
        // position of the token; lane j forms the rotation of pair j, then every lane fetches its four
        const int frame = (a.desc ? a.desc->frame_pos0[b] : st.frame_pos0) + i / a.tokens_per_frame;
        const int inside = i % a.tokens_per_frame;
        const int axis = a.pair_axis[lane];
        const int pos = axis == 0 ? frame : (axis == 1 ? inside / a.grid_w : inside % a.grid_w);
        double sn, cs;
        sincos((double)pos * a.inv_freq[lane], &sn, &cs);
        const float cf_own = (float)cs, sf_own = (float)sn;
        float cf[4], sf[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            cf[e] = __shfl(cf_own, p0 + e, kWave);
            sf[e] = __shfl(sf_own, p0 + e, kWave);
        }
        const long long g = (a.desc ? a.desc->g0[b] : st.g0) + i;
        const int slot = slot_of(g, a.S, a.W);
        if (lane == 0) st.ids[slot] = g;
        bf16* qo = a.q_out + (size_t)row * C;
#pragma unroll
        for (int it = 0; it < kMaxIt; ++it) {
            const int h = hl + 4 * it;
            if (h < a.H) {
                const int c = h * kHeadDim + 2 * p0;
                const f32x4 gq0 = *reinterpret_cast<const f32x4*>(a.g_q + c), gq1 = *reinterpret_cast<const f32x4*>(a.g_q + c + 4);
                const f32x4 gk0 = *reinterpret_cast<const f32x4*>(a.g_k + c), gk1 = *reinterpret_cast<const f32x4*>(a.g_k + c + 4);
                bf16x8 qr, kr;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float gqa = e < 2 ? gq0[2 * e] : gq1[2 * e - 4], gqb = e < 2 ? gq0[2 * e + 1] : gq1[2 * e - 3];
                    const float gka = e < 2 ? gk0[2 * e] : gk1[2 * e - 4], gkb = e < 2 ? gk0[2 * e + 1] : gk1[2 * e - 3];
                    const float q0 = (float)qv[it][2 * e] * rq * gqa, q1 = (float)qv[it][2 * e + 1] * rq * gqb;
                    const float k0 = (float)kv[it][2 * e] * rk * gka, k1 = (float)kv[it][2 * e + 1] * rk * gkb;
                    qr[2 * e] = (bf16)(q0 * cf[e] - q1 * sf[e]);
                    qr[2 * e + 1] = (bf16)(q0 * sf[e] + q1 * cf[e]);
                    kr[2 * e] = (bf16)(k0 * cf[e] - k1 * sf[e]);
                    kr[2 * e + 1] = (bf16)(k0 * sf[e] + k1 * cf[e]);
                }
                *reinterpret_cast<bf16x8*>(qo + c) = qr;
                *reinterpret_cast<bf16x8*>(st.k_cache + ((size_t)h * st.cap + slot) * kHeadDim + 2 * p0) = kr;
            }
        }
        return;
    }
    // ---- V^T tiles
    __shared__ bf16 tile[VT_TOK * VT_LD];
    const int vb = blockIdx.x - norm_blocks;
    const int h = vb % a.H;
    const int tile_id = vb / a.H;
    const int b = tile_id / tiles_per_stream;
    const int tok0 = (tile_id - b * tiles_per_stream) * VT_TOK;
    const AppendStream& st = a.st[b];
    // read: 64 tokens x 128 channels, 16-byte chunks, stored to LDS as 4-byte words
    for (int idx = threadIdx.x; idx < VT_TOK * 16; idx += 256) {
        const int tok = idx >> 4, c = idx & 15;
        if (tok0 + tok < a.L) {
            const bf16* vp = a.qkv + ((size_t)b * a.L + tok0 + tok) * 3 * C + 2 * C + h * kHeadDim + c * 8;
            const bf16x8 v = *reinterpret_cast<const bf16x8*>(vp);
            bf16x2* dst = reinterpret_cast<bf16x2*>(tile + tok * VT_LD + c * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[e] = bf16x2{v[2 * e], v[2 * e + 1]};
        }
    }
    __syncthreads();
    // write: lane = token, each wave takes 32 of the 128 channels
    const int tok = lane;
    if (tok0 + tok < a.L) {
        const int slot = slot_of((a.desc ? a.desc->g0[b] : st.g0) + tok0 + tok, a.S, a.W);
        bf16* vo = st.vt_cache + (size_t)h * kHeadDim * st.cap + vt_column(slot);
        for (int d = wave * 32; d < wave * 32 + 32; ++d) vo[(size_t)d * st.cap] = tile[tok * VT_LD + d];
    }
}

// ------------------------------------------------------------------ plain append of final rows
__global__ __launch_bounds__(256) void plain_append_kernel(PlainAppendArgs a, int k_blocks) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int C = a.C;
    if ((int)blockIdx.x < k_blocks) {
        const int row = blockIdx.x * 4 + wave;
        if (row >= a.n) return;
        const long long g = a.st.g0 + row;
        const int slot = slot_of(g, a.S, a.W);
        if (lane == 0 && a.st.ids != nullptr) a.st.ids[slot] = g;
        for (int h = 0; h < a.H; ++h) {
            const bf16x2 kv = *reinterpret_cast<const bf16x2*>(a.k + (size_t)row * C + h * kHeadDim + 2 * lane);
            *reinterpret_cast<bf16x2*>(a.st.k_cache + ((size_t)h * a.st.cap + slot) * kHeadDim + 2 * lane) = kv;
        }
        return;
    }
    __shared__ bf16 tile[VT_TOK * VT_LD];
    const int vb = blockIdx.x - k_blocks;
    const int h = vb % a.H;
    const int tok0 = (vb / a.H) * VT_TOK;
    for (int idx = threadIdx.x; idx < VT_TOK * 16; idx += 256) {
        const int tok = idx >> 4, c = idx & 15;
        if (tok0 + tok < a.n) {
            const bf16x8 v = *reinterpret_cast<const bf16x8*>(a.v + (size_t)(tok0 + tok) * C + h * kHeadDim + c * 8);
            bf16x2* dst = reinterpret_cast<bf16x2*>(tile + tok * VT_LD + c * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[e] = bf16x2{v[2 * e], v[2 * e + 1]};
        }
    }
    __syncthreads();
    const int tok = lane;
    if (tok0 + tok < a.n) {
        const int slot = slot_of(a.st.g0 + tok0 + tok, a.S, a.W);
        bf16* vo = a.st.vt_cache + (size_t)h * kHeadDim * a.st.cap + vt_column(slot);
        for (int d = wave * 32; d < wave * 32 + 32; ++d) vo[(size_t)d * a.st.cap] = tile[tok * VT_LD + d];
    }
}

// ------------------------------------------------------------------ conditioning
struct TimestepArgs {
    float t[kMaxBatch];
};

__global__ void timestep_embedding_kernel(TimestepArgs ts, const StepDesc* desc, float* emb, int B, int t_dim,
                                          double log2_base) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * t_dim) return;
    const int b = idx / t_dim;
    const int j = idx - b * t_dim;
    const int half = t_dim / 2;
    const int jj = j < half ? j : j - half;
    const double w = exp2(-log2_base * (double)jj / (double)half);
    const double arg = (double)(desc ? desc->timestep[b] : ts.t[b]) * w;
    emb[idx] = (float)(j < half ? cos(arg) : sin(arg));
}

// one wave per output n; the B input rows reuse each weight row
__global__ __launch_bounds__(256) void gemv_kernel(const float* x, const bf16* w, const float* bias, float* y, int B,
                                                   int N, int K, int silu_in) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    float acc[kMaxBatch];
#pragma unroll
    for (int b = 0; b < kMaxBatch; ++b) acc[b] = 0.0f;
    const bf16* wp = w + (size_t)n * K;
    for (int k = lane * 8; k < K; k += 64 * 8) {
        const bf16x8 wv = *reinterpret_cast<const bf16x8*>(wp + k);
#pragma unroll
        for (int b = 0; b < kMaxBatch; ++b) {
            if (b < B) {
                const float* xp = x + (size_t)b * K + k;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float xv = xp[e];
                    if (silu_in) xv = silu_f(xv);
                    acc[b] += xv * (float)wv[e];
                }
            }
        }
    }
#pragma unroll
    for (int b = 0; b < kMaxBatch; ++b) {
        if (b < B) {
            const float s = wave_sum(acc[b]);
            if (lane == 0) y[(size_t)b * N + n] = s + bias[n];
        }
    }
}

}  // namespace

template <bool EARLY>
static hipError_t launch_layernorm_t(const LnArgs& a, hipStream_t s) {
    const dim3 grid((a.rows + 1) / 2), block(256);
    const int nv = (a.C + 511) / 512;                   // float4 values per lane: 128 lanes per row
    if (nv <= 1) hipLaunchKernelGGL((layernorm_kernel<1, EARLY>), grid, block, 0, s, a);
    else if (nv <= 3) hipLaunchKernelGGL((layernorm_kernel<3, EARLY>), grid, block, 0, s, a);
    else if (nv <= 4) hipLaunchKernelGGL((layernorm_kernel<4, EARLY>), grid, block, 0, s, a);
    else if (nv <= 6) hipLaunchKernelGGL((layernorm_kernel<6, EARLY>), grid, block, 0, s, a);
    else if (nv <= 10) hipLaunchKernelGGL((layernorm_kernel<10, EARLY>), grid, block, 0, s, a);
    else if (nv <= 16) hipLaunchKernelGGL((layernorm_kernel<16, EARLY>), grid, block, 0, s, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_layernorm(const LnArgs& a, hipStream_t s) {
    return a.rows <= 4096 ? launch_layernorm_t<true>(a, s) : launch_layernorm_t<false>(a, s);
}

hipError_t launch_rmsnorm_inplace(bf16* x, const float* gain, int rows, int C, int ld, float eps, hipStream_t s) {
    const dim3 grid((rows + 3) / 4), block(256);
    const int nv = (C + 511) / 512;                     // 16-byte pieces per lane
    if (nv <= 1) hipLaunchKernelGGL(rmsnorm_inplace_kernel<1>, grid, block, 0, s, x, gain, rows, C, ld, eps);
    else if (nv <= 3) hipLaunchKernelGGL(rmsnorm_inplace_kernel<3>, grid, block, 0, s, x, gain, rows, C, ld, eps);
    else if (nv <= 6) hipLaunchKernelGGL(rmsnorm_inplace_kernel<6>, grid, block, 0, s, x, gain, rows, C, ld, eps);
    else if (nv <= 10) hipLaunchKernelGGL(rmsnorm_inplace_kernel<10>, grid, block, 0, s, x, gain, rows, C, ld, eps);
    else if (nv <= 16) hipLaunchKernelGGL(rmsnorm_inplace_kernel<16>, grid, block, 0, s, x, gain, rows, C, ld, eps);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_rope_append(const RopeAppendArgs& a, hipStream_t s) {
    const int norm_blocks = (a.B * a.L + 3) / 4;
    const int tiles_per_stream = (a.L + VT_TOK - 1) / VT_TOK;
    const int v_blocks = a.B * tiles_per_stream * a.H;
    hipLaunchKernelGGL(rope_append_kernel, dim3(norm_blocks + v_blocks), dim3(256), 0, s, a, norm_blocks,
                       tiles_per_stream);
    return hipGetLastError();
}

hipError_t launch_plain_append(const PlainAppendArgs& a, hipStream_t s) {
    const int k_blocks = (a.n + 3) / 4;
    const int v_blocks = ((a.n + VT_TOK - 1) / VT_TOK) * a.H;
    hipLaunchKernelGGL(plain_append_kernel, dim3(k_blocks + v_blocks), dim3(256), 0, s, a, k_blocks);
    return hipGetLastError();
}

hipError_t launch_text_relayout(const bf16* k_rows, const bf16* v_rows, bf16* kt, bf16* vtt, int L_t, int C, int H,
                                int cap, hipStream_t s) {
    // the text K/V buffers are a cache with no ring: slot = token index
    PlainAppendArgs a;
    a.k = k_rows;
    a.v = v_rows;
    a.n = L_t;
    a.C = C;
    a.H = H;
    a.S = cap;          // every token is "sink": slot(g) = g
    a.W = 1;
    a.st.k_cache = kt;
    a.st.vt_cache = vtt;
    a.st.ids = nullptr;
    a.st.g0 = 0;
    a.st.frame_pos0 = 0;
    a.st.cap = cap;
    return launch_plain_append(a, s);
}

hipError_t launch_gemv(const float* x, const bf16* w, const float* bias, float* y, int B, int N, int K, int silu_in,
                       hipStream_t s) {
    hipLaunchKernelGGL(gemv_kernel, dim3((N + 3) / 4), dim3(256), 0, s, x, w, bias, y, B, N, K, silu_in);
    return hipGetLastError();
}

hipError_t launch_timestep_embedding(const float* t_host, const StepDesc* desc, float* emb, int B, int t_dim, double base,
                                     hipStream_t s) {
    TimestepArgs ts;
    for (int b = 0; b < kMaxBatch; ++b) ts.t[b] = (t_host && b < B) ? t_host[b] : 0.0f;
    const int n = B * t_dim;
    hipLaunchKernelGGL(timestep_embedding_kernel, dim3((n + 255) / 256), dim3(256), 0, s, ts, desc, emb, B, t_dim,
                       log2(base));
    return hipGetLastError();
}

namespace {
__global__ void set_step_desc_kernel(StepDesc d, StepDesc* dst) {
    if (threadIdx.x == 0) *dst = d;
}
}  // namespace

hipError_t launch_set_step_desc(const StepDesc& d, StepDesc* dst, hipStream_t s) {
    hipLaunchKernelGGL(set_step_desc_kernel, dim3(1), dim3(64), 0, s, d, dst);
    return hipGetLastError();
}

}  // namespace sdv2
