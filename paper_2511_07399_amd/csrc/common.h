// Internal declarations shared by the HIP sources of libsdv2 (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sdv2 {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kHeadDim = 128;
constexpr int kMaxBatch = 8;
constexpr int kLatentChannels = 16;      // VAE latent channels; a token covers 2 x 2 latent positions (64 numbers)

// Column of a V^T cache row that holds slot s: inside every group of 16 slots the two middle groups of four
// trade places (0-3, 8-11, 4-7, 12-15), the order in which the S^T accumulator of the attention kernel holds
// its keys.  The map is its own inverse.
__host__ __device__ __forceinline__ int vt_column(int s) { return (s & ~12) | ((s & 4) << 1) | ((s & 8) >> 1); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float gelu_tanh_f(float x) {
    // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3).  The exponent is formed
    // directly in base 2 and the quotient is x times the hardware reciprocal (1 ulp): the caller rounds the
    // result to bf16.
    constexpr float k1 = -2.0f * 1.4426950408889634f * 0.7978845608028654f;
    constexpr float k3 = k1 * 0.044715f;
    const float e = __builtin_amdgcn_exp2f(x * fmaf(x * x, k3, k1));
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ---------------------------------------------------------------- launchers (host side)
enum GemmEpilogue { kEpiBias = 0, kEpiBiasGelu = 1, kEpiGatedResidual = 2, kEpiResidual = 3,
                    kEpiPartial = 4 /* internal: fp32 partial sums of one k part, no bias */ };

struct GemmArgs {
    const bf16* a;        // [M, K]
    const bf16* w;        // [N, K]
    const float* bias;    // [N] or null
    void* out;            // bf16 [M, N] (epilogue 0, 1) or fp32 [M, N] (2, 3)
    int M, N, K;
    int epilogue;
    const float* gate_a;  // [N]
    const float* gate_b;  // [(M / rows_per_gate), gate_b_stride]
    int gate_b_stride;
    int rows_per_gate;
    // Optional scratch for shapes whose plan splits the k range over several workgroups per tile (null: never
    // split): room for splitk_floats fp32 partial sums.  A second, elementwise kernel adds the parts in k order
    // and applies the epilogue, so the result does not depend on scheduling.
    float* splitk_partials;
    size_t splitk_floats;
};
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);
// fp32 partial sums the planned launch of an [M, K] x [N, K] product needs (0: its plan does not split k)
size_t gemm_splitk_floats(int M, int N, int K, int epilogue);
// Name of the kernel instantiation the plan picks for a shape, spelled as a profiler prints it (benchmark only).
void gemm_plan_name(int M, int N, int K, int epilogue, char* out, size_t cap);
// Tuning hooks (tests and sweeps): a tile plan that replaces the planner's for every shape; false if not understood.
bool set_gemm_tile_override(const char* spec);

// What changes from one denoising step to the next, kept in device memory when the step is replayed from a captured
// graph (the kernels then read it from there instead of from their by-value arguments).
struct StepDesc {
    long long g0[kMaxBatch];          // token id of the chunk's first token, per stream of the call
    int frame_pos0[kMaxBatch];        // RoPE frame index of the chunk's first frame
    int kv_len[kMaxBatch];            // resident slots after the append
    float timestep[kMaxBatch];
};

struct AttnArgs {
    const bf16* q;                    // [B, L, C]
    const bf16* k[kMaxBatch];         // [H][cap][128]
    const bf16* vt[kMaxBatch];        // [H][128][cap]
    int kv_len[kMaxBatch];
    int cap[kMaxBatch];
    bf16* o;                          // [B, L, C]
    int B, L, H;
    float* part_o;                    // workspace: [splits][B*L][C] fp32
    float* part_ml;                   // workspace: [splits][B*L][H][2] fp32
    int splits;                       // chosen by attention_plan
    const StepDesc* desc;             // null: kv_len above; else kv_len is read from the device descriptor
};
int attention_plan_splits(int B, int L, int H, int max_kv_len);
// Tuning hooks: waves per workgroup (4, 8; 0 = planner) and key-range splits (0 = planner); -1 leaves a value as is.
void set_attention_overrides(int waves, int splits);
size_t attention_workspace_bytes(int B, int L, int C, int max_kv_len);
hipError_t launch_attention(const AttnArgs& a, hipStream_t s, int part = 0);   // part 1: the kernel; 2: the merge pass only
bool attention_has_merge_pass(const AttnArgs& a);
void attention_plan_name(const AttnArgs& a, char* out, size_t cap);      // only B, L, H, kv_len and cap are read

// LayerNorm over C with an affine that is either adaLN modulation or a plain (gamma, beta).
struct LnArgs {
    const float* x;       // [rows, C]
    bf16* out;            // [rows, C]
    int rows, C;
    float eps;
    // scale = 1 + (scale_a[c] + scale_b[stream * b_stride + c]) when modulated, gamma[c] otherwise
    const float* scale_a;
    const float* scale_b; // null: plain affine (scale_a = gamma, shift_a = beta)
    const float* shift_a;
    const float* shift_b;
    int b_stride;
    int rows_per_stream;
};
hipError_t launch_layernorm(const LnArgs& a, hipStream_t s);

// launch_gemm for a residual epilogue (2 or 3) whose output x is the input of a LayerNorm that follows it: when the
// plan splits k, the pass that adds the parts owns whole rows and also writes that LayerNorm's output (ln.x is
// ignored: the rows are g.out's; ln.rows = g.M, ln.C = g.N).  *ln_done tells whether it did; if not, the caller
// launches the LayerNorm itself.
// part 0: everything; 1: only the kernel on the matrix cores; 2: only the pass that adds the k parts.
hipError_t launch_gemm_then_layernorm(const GemmArgs& g, const LnArgs& ln, bool* ln_done, hipStream_t s, int part = 0);
hipError_t launch_gemm_part(const GemmArgs& g, hipStream_t s, int part);
bool gemm_splits_k(const GemmArgs& g);               // whether the planned launch has such a second pass

// In-place RMSNorm over C of bf16 rows, times gain.
hipError_t launch_rmsnorm_inplace(bf16* x, const float* gain, int rows, int C, int ld, float eps, hipStream_t s);

// q/k RMSNorm + 3D-RoPE + append of k and v into the rolling cache.
struct AppendStream {
    bf16* k_cache;        // [H][cap][128]
    bf16* vt_cache;       // [H][128][cap]
    long long* ids;       // [cap]
    long long g0;         // token id of the chunk's first token
    int frame_pos0;
    int cap;
};
struct RopeAppendArgs {
    const bf16* qkv;      // [B*L, 3C]   (or separate k, v when q_out == null)
    bf16* q_out;          // [B*L, C]
    const float* g_q;
    const float* g_k;
    int B, L, C, H;
    int tokens_per_frame, grid_w;
    int S, W;
    float eps;
    double inv_freq[kHeadDim / 2];    // rotation frequency of each pair of a head
    int pair_axis[kHeadDim / 2];      // 0 frame, 1 row, 2 col
    AppendStream st[kMaxBatch];
    const StepDesc* desc;             // null: g0 and frame_pos0 of st[]; else they are read from the device descriptor
};
hipError_t launch_rope_append(const RopeAppendArgs& a, hipStream_t s);

// Plain append of final k, v rows [n, C] (standalone cache call).
struct PlainAppendArgs {
    const bf16* k;        // [n, C]
    const bf16* v;        // [n, C]
    int n, C, H, S, W;
    AppendStream st;
};
hipError_t launch_plain_append(const PlainAppendArgs& a, hipStream_t s);

// Sink refresh and RoPE refresh of one (layer, stream) cache (Section 4.1).
struct SinkSimArgs {
    const bf16* vt;       // [H][128][cap]
    int H, cap, P;        // P = tokens per frame
    int src0;             // first slot of the frame h_t
    int m;                // sink frames; sink frame i starts at slot i * P
    float* partial;       // [m][blocks][3] fp32
    float* alpha;         // [m]
};
int sink_similarity_blocks(int H);
hipError_t launch_sink_similarity(const SinkSimArgs& a, hipStream_t s);
struct SinkCopyArgs {
    bf16* k;              // [H][cap][128]
    bf16* vt;             // [H][128][cap]
    long long* ids;       // [cap]
    int H, cap, P;
    int src0, dst0;       // first slots of the source frame and of the sink frame
};
hipError_t launch_refresh_sink(const SinkCopyArgs& a, hipStream_t s);
constexpr int kMaxFramePairs = kHeadDim / 2;
struct RotateKeysArgs {
    bf16* k;              // [H][cap][128]
    int H, cap, S;
    int sink_fill;        // filled sink slots [0, sink_fill)
    int n_slots;          // sink_fill + filled window slots [S, S + n_slots - sink_fill)
    int n_pairs;          // leading pairs of a head that belong to the frame axis
    float cs[kMaxFramePairs], sn[kMaxFramePairs];
};
hipError_t launch_rotate_keys(const RotateKeysArgs& a, hipStream_t s);

// Motion-aware noise scheduler (Section 4.1).  Device state: kMotionHeaderFloats header floats (s, frame count as
// int bits), then the ring of the last k + 1 intensities, then kMotionMaxFrames * kMotionBlocks partial sums.
constexpr int kMotionHeaderFloats = 16;
constexpr int kMotionBlocks = 64;
constexpr int kMotionMaxFrames = 16;
constexpr int kMotionMaxK = 1023;
struct MotionArgs {
    const float* frames;   // [T][n]
    const float* prev;     // [n] or null: the frame before frames[0]
    long long n;
    int T, k, vec4;
    float sigma, lambda, s_min, s_max;
    float* state;
    float* partial;        // [T][kMotionBlocks]
    float* d_out;          // [T]
    float* dhat_out;       // [T]
    float* s_out;          // [T]
};
hipError_t launch_motion_init(float* state, int n_floats, float s_init, hipStream_t s);
hipError_t launch_motion_update(const MotionArgs& a, hipStream_t s);

// Re-layout of text K/V rows [L_t, C] into the cache layouts.
hipError_t launch_text_relayout(const bf16* k_rows, const bf16* v_rows, bf16* kt, bf16* vtt,
                                int L_t, int C, int H, int cap, hipStream_t s);

// y[b][n] = act_out(sum_k act_in(x[b][k]) W[n][k] + bias[n]); x, y fp32; W bf16 [N, K]; B <= kMaxBatch.
hipError_t launch_gemv(const float* x, const bf16* w, const float* bias, float* y, int B, int N, int K,
                       int silu_in, hipStream_t s);
// t_host: the B timesteps (by value into the launch), or null with desc: they are read from the device descriptor
hipError_t launch_timestep_embedding(const float* t_host, const StepDesc* desc, float* emb, int B, int t_dim, double base,
                                     hipStream_t s);
hipError_t launch_set_step_desc(const StepDesc& d, StepDesc* dst, hipStream_t s);
// While set (per thread), the dense launchers only make sure their kernels' attributes are set and launch nothing:
// used once before a stream capture so that no attribute call falls inside it.
void set_attributes_only(bool on);
bool attributes_only();

// Latents <-> tokens, noise rate, sampler update (latent_io.hip).  z, v: fp32 [B][16][F][2 gh][2 gw]; patches bf16 and
// tok fp32 [B F gh gw][64]; n = elements per stream; rate / sigma / sigma_next: host arrays [B].
hipError_t launch_patchify(const float* z, bf16* patches, int B, int F, int gh, int gw, hipStream_t s);
hipError_t launch_unpatchify(const float* tok, float* v, int B, int F, int gh, int gw, hipStream_t s);
hipError_t launch_noise(const float* x, const float* eps, float* out, int B, long long n, const float* rate, hipStream_t s);
hipError_t launch_sampler(const float* z, const float* v, const float* eps, float* z_next, float* x0, int B, long long n,
                          const float* sigma, const float* sigma_next, hipStream_t s);

// Benchmark-only microkernels: a register-resident loop of bf16 matrix instructions (iters x 8 per wave, eight waves
// per workgroup) and a streaming copy of `bytes` (multiple of 16) bytes.
hipError_t launch_peak_mfma(int iters, int workgroups, float* sink, hipStream_t s);
double peak_mfma_flops(int iters, int workgroups);
hipError_t launch_peak_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
hipError_t launch_peak_lds(int iters, const unsigned char* src, float* sink, unsigned long long* ticks, hipStream_t s);

}  // namespace sdv2
