/*
 * sdv2.h - C ABI of libsdv2: the streaming causal video-DiT block for one chunk
 * on one MI355X (gfx950), with a sink-token-guided rolling KV cache.
 *
 * The calls follow StreamDiffusionV2's statement of the streaming problem: an
 * unbounded sequence of short chunks per stream (Section 1, "Efficiency
 * objectives"; Section 3), each denoised in 1-4 steps (Section 5.1) by a causal
 * DiT (Section 5.1 "Models") against a per-layer cache made of sink tokens and
 * a rolling window of recent frames that is updated frame by frame (abstract;
 * Section 1; Appendix D, rolling-KV-cache figure), with B independent streams
 * batched through one forward (Section 4.1, SLO-aware batching scheduler).
 * The per-layer work is the one Appendix B costs: projections and FFN
 * (24 b L_q C^2 flops) and attention over the cache (4 b L_q L_kv C flops).
 *
 * General rules
 *  - Every function returns 0 (SDV2_OK) or a negative sdv2_status; the text of
 *    the last error of the calling thread is at sdv2_last_error().
 *  - All arguments are validated before anything is launched or any state is
 *    changed: a failed call leaves cache state and device memory untouched.
 *  - "dev" pointers are device memory owned by the caller; "host" pointers are
 *    ordinary host memory.  The library never allocates or frees device memory
 *    and never synchronises: work is enqueued on the caller's hipStream_t
 *    (passed as void*; NULL is the default stream).
 *  - Matrices are bf16, row-major, stored [out, in] (y = x W^T + b); vectors
 *    (biases, gains, modulation tables) are fp32.  The hidden state x is fp32.
 *  - Head h owns columns [h*128, (h+1)*128) of a token row; head_dim is 128.
 *  - Calls that touch the same cache, x or workspace must be ordered by the
 *    caller (same stream); ring positions are tracked on the host in call order.
 */
#ifndef SDV2_H
#define SDV2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SDV2_MAX_BATCH 8      /* streams per dit_block_forward / denoise_step call */
#define SDV2_HEAD_DIM 128

typedef enum sdv2_status {
    SDV2_OK = 0,
    SDV2_INVALID_ARG = -1,          /* null pointer, bad size, size not a multiple of what is required */
    SDV2_BAD_STATE = -2,            /* e.g. advance = 0 without a previous append of the same size */
    SDV2_WORKSPACE_TOO_SMALL = -3,
    SDV2_HIP_ERROR = -4             /* a launch failed; the text names the HIP error */
} sdv2_status;

/* Shape of the model.  Set struct_size = sizeof(sdv2_model_cfg). */
typedef struct sdv2_model_cfg {
    uint32_t struct_size;
    int32_t C;            /* model width, = n_heads * 128, multiple of 128, <= 8192 */
    int32_t n_heads;
    int32_t ffn_dim;      /* multiple of 128 */
    int32_t grid_h;       /* token rows per latent frame */
    int32_t grid_w;       /* token columns per latent frame; tokens_per_frame = grid_h * grid_w */
    int32_t text_len;     /* text tokens L_t (> 0) */
    int32_t n_layers;
    int32_t t_dim;        /* width of the sinusoidal timestep embedding (even, multiple of 8; 256) */
    float eps;            /* LayerNorm / RMSNorm epsilon (1e-6) */
    float rope_base;      /* 10000 */
} sdv2_model_cfg;

/* Shape of the cache.  All capacities in tokens and whole frames. */
typedef struct sdv2_cache_cfg {
    uint32_t struct_size;
    int32_t n_layers;
    int32_t n_streams;
    int32_t n_heads;
    int32_t tokens_per_frame;
    int32_t sink_tokens;      /* S >= 0: the first S tokens of a stream, never evicted */
    int32_t window_tokens;    /* W > 0: ring of the most recent tokens, the current chunk included */
} sdv2_cache_cfg;

/* One layer's parameters (all dev pointers). */
typedef struct sdv2_block_weights {
    uint32_t struct_size;
    uint32_t reserved;
    const void* W_qkv;        /* bf16 [3C, C]: rows 0..C-1 = W_q, C..2C-1 = W_k, 2C..3C-1 = W_v */
    const float* b_qkv;       /* [3C] */
    const float* g_q;         /* [C] RMSNorm gain of q (norm over all C) */
    const float* g_k;         /* [C] */
    const void* W_o;          /* bf16 [C, C] */
    const float* b_o;         /* [C] */
    const float* mod_table;   /* [6, C]: shift1, scale1, gate1, shift2, scale2, gate2 (added to e0) */
    const float* ln3_gamma;   /* [C] affine LayerNorm before the cross-attention */
    const float* ln3_beta;    /* [C] */
    const void* W_cq;         /* bf16 [C, C] */
    const float* b_cq;        /* [C] */
    const float* g_cq;        /* [C] */
    const void* W_ck;         /* bf16 [C, C]  (used by sdv2_text_kv_prepare only) */
    const float* b_ck;
    const float* g_ck;
    const void* W_cv;         /* bf16 [C, C]  (used by sdv2_text_kv_prepare only) */
    const float* b_cv;
    const void* W_co;         /* bf16 [C, C] */
    const float* b_co;
    const void* W_1;          /* bf16 [F, C] */
    const float* b_1;         /* [F] */
    const void* W_2;          /* bf16 [C, F] */
    const float* b_2;         /* [C] */
} sdv2_block_weights;

/* Whole-model parameters. */
typedef struct sdv2_model_weights {
    uint32_t struct_size;
    uint32_t reserved;
    const sdv2_block_weights* blocks;   /* host array [n_layers] */
    const void* W_t1;         /* bf16 [C, t_dim] */
    const float* b_t1;        /* [C] */
    const void* W_t2;         /* bf16 [C, C] */
    const float* b_t2;        /* [C] */
    const void* W_mod;        /* bf16 [6C, C] */
    const float* b_mod;       /* [6C] */
} sdv2_model_weights;

/* What one stream contributes to a batched call. */
typedef struct sdv2_chunk_desc {
    int32_t stream_id;        /* which cache stream; distinct within one call */
    int32_t frame_pos0;       /* RoPE frame index of the chunk's first frame (caller's policy) */
    int32_t n_frames;         /* frames in the chunk; the same for every stream of a call */
    int32_t advance;          /* 1: a new chunk (appends, evicts); 0: a further denoising step of the
                                 chunk appended last (overwrites its K/V in place) */
} sdv2_chunk_desc;

/* Host-side view of one (layer, stream) cache; compared bit for bit in the tests. */
typedef struct sdv2_cache_state {
    int64_t total;            /* tokens ever appended */
    int64_t evicted;          /* tokens that have left the window */
    int32_t sink_fill;
    int32_t win_fill;
    int32_t oldest_slot;      /* physical slot of the oldest window token, -1 if the window is empty */
    int32_t next_slot;        /* physical slot the next token will take */
} sdv2_cache_state;

typedef struct sdv2_kv_cache sdv2_kv_cache;   /* opaque host handle */

const char* sdv2_last_error(void);
int32_t sdv2_version(void);

/* ------------------------------------------------------------------------------------------------
 * Rolling KV cache (abstract; Section 1; Appendix D rolling-KV-cache figure).
 *
 * Token g (0-based count of tokens ever appended to a stream's layer) lives in physical slot
 *     slot(g) = g                      if g < S        (sink: written once, never evicted)
 *               S + (g - S) mod W      otherwise       (ring: a token leaves when a later one
 *                                                       lands on its slot, i.e. first in first out)
 * Resident tokens always occupy the slot prefix [0, min(total, S + W)).
 *
 * Device layout per (layer, stream), cap = S + W rounded up to a multiple of 64:
 *     K    bf16 [n_heads][cap][128]      (post-RMSNorm, post-RoPE keys)
 *     V^T  bf16 [n_heads][128][cap]      (values transposed; slot s sits in column
 *                                         (s & ~12) | ((s & 4) << 1) | ((s & 8) >> 1): inside every group of 16
 *                                         slots the two middle groups of four trade places, which is the key
 *                                         order of the attention kernel's accumulators)
 *     ids  int64 [cap]                   (token id held by each slot, written by the append kernel;
 *                                         meaningful only for slots < min(total, S + W))
 * ------------------------------------------------------------------------------------------------ */

/* Bytes of device storage the caller must provide for the whole cache (0 on bad cfg). */
size_t sdv2_kv_cache_bytes(const sdv2_cache_cfg* cfg);

/* Create a handle over caller-owned storage `dev_storage` (256-byte aligned, `bytes` long, must
 * outlive the handle).  All streams start empty.  Nothing is launched; storage is not cleared.
 * Errors: null pointers, S < 0, W <= 0, S or W not a multiple of tokens_per_frame, bytes too small. */
int32_t sdv2_kv_cache_init(const sdv2_cache_cfg* cfg, void* dev_storage, size_t bytes, sdv2_kv_cache** out);

/* Free the host handle only. */
int32_t sdv2_kv_cache_destroy(sdv2_kv_cache* cache);

/* Forget one stream (all layers): total = 0.  Host-only. */
int32_t sdv2_kv_cache_reset(sdv2_kv_cache* cache, int32_t stream_id);

/* Append n_tokens final keys/values (dev, bf16 [n_tokens, C], already normalised and rotated).
 * advance = 1: the tokens get ids [total, total + n_tokens), total grows, the oldest window tokens
 *              that no longer fit are evicted (overwritten).
 * advance = 0: rewrites the values of the most recent append in place; needs the same n_tokens
 *              (else SDV2_BAD_STATE).
 * Errors: n_tokens <= 0, > W, or not a multiple of tokens_per_frame; bad layer / stream.
 * sdv2_dit_block_forward performs the identical state transition with its fused kernel. */
int32_t sdv2_kv_cache_append_evict(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id,
                                   const void* k_dev, const void* v_dev, int32_t n_tokens,
                                   int32_t advance, void* hip_stream);

/* Host-side state and slot map (no device access, no synchronisation).
 * slot_map_out: host int64 [S + W]; token id per slot, -1 where nothing is resident. */
int32_t sdv2_kv_cache_state(const sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, sdv2_cache_state* out);
int32_t sdv2_kv_cache_slot_map(const sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int64_t* slot_map_out);

/* Device addresses of one (layer, stream) cache and its padded capacity (for read-back in tests). */
int32_t sdv2_kv_cache_device_ptrs(const sdv2_kv_cache* cache, int32_t layer, int32_t stream_id,
                                  void** k_dev, void** vt_dev, int64_t** ids_dev, int32_t* cap);

/* ------------------------------------------------------------------------------------------------
 * Adaptive sink refresh and RoPE refresh (Section 4.1, "Adaptive sink and RoPE refresh").
 *
 * The section defines, for sinks s_1 .. s_m and a new chunk embedding h_t:  alpha_i = cos(h_t, s_i);  s_i is kept
 * when alpha_i >= tau and replaced by h_t otherwise; and, past a frame index T_reset, the rotary phase of frame t
 * is that of frame t - T_reset.  It does not say what the vectors are; this library takes, per (layer, stream):
 *   s_i  = sink frame i of the cache (tokens_per_frame slots starting at slot i * tokens_per_frame;
 *          m = sink_tokens / tokens_per_frame),
 *   h_t  = one frame of the most recent append, frame_back = 0 being its last frame,
 *   cos  = cosine of the two frames' cached VALUE rows, each flattened to tokens_per_frame * C numbers (values
 *          carry no rotary phase),
 *   s_i <- h_t = a copy of that frame's cached keys, values and token ids into the sink frame's slots (the keys
 *          keep the phase of the frame they came from; until that frame leaves the window its tokens are
 *          resident twice).
 * The comparison with tau is the caller's: read alpha back and call sdv2_kv_cache_refresh_sink for the sinks to
 * replace, so that the host-side slot map stays a function of the call history.  The frame index handed to the
 * block (chunk_desc.frame_pos0) is the caller's as well; when it is lowered by delta frames the cached keys are
 * moved along with sdv2_kv_cache_rotate_keys, which keeps every query/key phase difference.
 *
 * sdv2_sink_similarity: alpha_dev (dev fp32 [m]) <- alpha_i.  fp32 partial sums per workgroup, added in double in a
 *   fixed order (deterministic).  Workspace: sdv2_sink_similarity_workspace_bytes(cache), 256-byte aligned.
 *   Errors: SDV2_BAD_STATE when the sink is not filled, nothing has been appended, or the frame asked for was
 *   itself stored in the sink; SDV2_INVALID_ARG for frame_back outside the latest append.
 * sdv2_kv_cache_refresh_sink: the copy, and the slot map's sink entries.  It closes the chunk: a later append with
 *   advance = 0 is refused (SDV2_BAD_STATE) until the next advancing append, because a repeated denoising step
 *   would rewrite the source frame but not its copy.  Same errors, plus sink_frame outside [0, m).
 * sdv2_kv_cache_rotate_keys: every resident key (sink and window) of the (layer, stream) cache is turned, in
 *   place, by -delta_frames * base^(-j / n_f) in each of the n_f = 22 leading pairs of a head (the frame axis of
 *   the 3-axis rotary embedding): a key cached at frame f becomes the key of frame f - delta_frames, rounded to
 *   bf16 again.  delta_frames may be negative.  Values, ids and all counters are untouched.
 * None of the three synchronises or allocates.
 * ------------------------------------------------------------------------------------------------ */
size_t sdv2_sink_similarity_workspace_bytes(const sdv2_kv_cache* cache);
int32_t sdv2_sink_similarity(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int32_t frame_back,
                             float* alpha_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream);
int32_t sdv2_kv_cache_refresh_sink(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int32_t sink_frame,
                                   int32_t frame_back, void* hip_stream);
int32_t sdv2_kv_cache_rotate_keys(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int32_t delta_frames,
                                  float rope_base, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Motion-aware noise scheduler (Section 4.1, "Motion-aware noise scheduler"), in the paper's notation:
 *   d_t    = sqrt( ||v_t - v_{t-1}||_2^2 / (C H W) )                      v_t: latent frame, C H W = frame_elems
 *   dhat_t = clip( max_{i in {t-k .. t}} d_i / sigma, 0, 1 )
 *   s_t    = lambda [ s_max - (s_max - s_min) dhat_t ] + (1 - lambda) s_{t-1}
 * Readings: the first frame of a stream has d = 0; the window is cut at the start of the stream; s before the
 * first frame is cfg.s_init.
 *
 * The recurrence lives in a small device buffer `state_dev` (sdv2_motion_state_bytes(cfg) bytes, 16-byte aligned,
 * one per stream, owned by the caller): sdv2_motion_init sets s = s_init and an empty window (one small kernel);
 * sdv2_motion_update consumes n_frames (1 .. 16) consecutive frames `frames_dev` (dev fp32 [n_frames][frame_elems])
 * and writes d_t, dhat_t and s_t of each to three dev fp32 [n_frames] arrays.  `prev_frame_dev` is the frame that
 * precedes frames_dev[0] (the last frame of the previous call), or NULL at the start of a stream.  fp32 arithmetic,
 * the sums of squares as fp32 partial sums per workgroup added in double in a fixed order (deterministic).
 * Calls on the same state must be ordered on one stream.  No allocation, no synchronisation.
 * Errors: bad cfg (k < 0 or > 1023, sigma <= 0, lambda outside (0, 1), s_min > s_max), null pointers, n_frames
 * outside 1 .. 16, frame_elems <= 0: SDV2_INVALID_ARG; state too small: SDV2_WORKSPACE_TOO_SMALL.
 * ------------------------------------------------------------------------------------------------ */
typedef struct sdv2_motion_cfg {
    uint32_t struct_size;
    int32_t k;            /* window: frames t-k .. t */
    float sigma;          /* normalising scale */
    float lambda;         /* update rate of the moving average, 0 < lambda < 1 */
    float s_min, s_max;   /* bounds of the noise rate */
    float s_init;         /* s before the first frame */
} sdv2_motion_cfg;
size_t sdv2_motion_state_bytes(const sdv2_motion_cfg* cfg);
int32_t sdv2_motion_init(const sdv2_motion_cfg* cfg, void* state_dev, size_t state_bytes, void* hip_stream);
int32_t sdv2_motion_update(const sdv2_motion_cfg* cfg, void* state_dev, size_t state_bytes, const float* frames_dev,
                           const float* prev_frame_dev, int32_t n_frames, int64_t frame_elems, float* d_out_dev,
                           float* dhat_out_dev, float* s_out_dev, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * SLO-aware batching scheduler (Section 4.1, "SLO-aware batching scheduler").  Host-only, no GPU work.
 * With T = frames_per_chunk frames per iteration for each of B batch slots and measured latencies L(T, B), the
 * achieved frequency is f = B T / L(T, B); B T must not exceed the frames already collected.  Given the caller's table
 * (batch_sizes[i], latency_s[i]), i < n (any order, sizes distinct), the call returns in *batch_out
 *   - the SMALLEST allowed size that meets f >= f_slo and whose f is within the fraction knee_tol (0 <= knee_tol < 1)
 *     of the best f among the sizes that meet it (the knee: beyond it a larger batch only adds latency), with
 *     *meets_slo_out = 1;
 *   - if no allowed size meets f_slo, the allowed size with the highest f (the smaller on ties), *meets_slo_out = 0;
 *   - 0 if no size is allowed (fewer than the smallest B T frames collected).
 * *frequency_out (optional) receives f of the returned size.  The latencies are the caller's measurements (e.g. of
 * sdv2_denoise_step); the paper's model L = (A(T, B) + P_model) / (eta BW_HBM) is not assumed.
 * Errors: null pointers, n <= 0, frames_per_chunk <= 0, a batch size < 1, a latency <= 0, knee_tol outside [0, 1).
 * ------------------------------------------------------------------------------------------------ */
int32_t sdv2_slo_pick_batch(const int32_t* batch_sizes, const double* latency_s, int32_t n, int32_t frames_per_chunk,
                            double f_slo, int64_t frames_collected, double knee_tol, int32_t* batch_out,
                            double* frequency_out, int32_t* meets_slo_out);

/* ------------------------------------------------------------------------------------------------
 * Text keys/values of the cross-attention (per prompt and layer; off the per-chunk path: prompt
 * changes are events, Section 1 "Vision quality objectives").
 *   K_t = RMSNorm(ctx W_ck^T + b_ck) g_ck,   V_t = ctx W_cv^T + b_cv
 * Output layout matches the cache: K_t bf16 [n_heads][cap_t][128], V_t^T bf16 [n_heads][128][cap_t],
 * cap_t = text_len rounded up to 64.  sdv2_text_kv_bytes gives the bytes of EACH of the two buffers.
 * ctx_dev: bf16 [text_len, C].  Workspace: sdv2_text_kv_workspace_bytes.
 * ------------------------------------------------------------------------------------------------ */
size_t sdv2_text_kv_bytes(const sdv2_model_cfg* cfg);
size_t sdv2_text_kv_workspace_bytes(const sdv2_model_cfg* cfg);
int32_t sdv2_text_kv_prepare(const sdv2_model_cfg* cfg, const sdv2_block_weights* w, const void* ctx_dev,
                             void* kt_dev, void* vtt_dev, void* workspace_dev, size_t workspace_bytes,
                             void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Timestep conditioning, once per denoising step:
 *   tvec = W_t2 SiLU(W_t1 emb(t) + b_t1) + b_t2,  emb(t) = [cos(t w_j) | sin(t w_j)], w_j = base^(-j/(t_dim/2))
 *   e0   = W_mod SiLU(tvec) + b_mod            -> dev fp32 [B, 6, C]
 * Exactly one of timesteps_host (host float [B]) and tvec_dev (dev fp32 [B, C]) is non-null; with
 * tvec_dev the first line is skipped.  Workspace: sdv2_conditioning_workspace_bytes(cfg, B).
 * ------------------------------------------------------------------------------------------------ */
size_t sdv2_conditioning_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B);
int32_t sdv2_conditioning(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, int32_t B,
                          const float* timesteps_host, const float* tvec_dev, float* e0_dev,
                          void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * One causal DiT block on one chunk of B streams (the per-layer work costed in Appendix B):
 *   (shift1, scale1, gate1, shift2, scale2, gate2) = mod_table + e0[b]
 *   h = LN(x)(1 + scale1) + shift1;  q, k, v = h W_qkv^T + b_qkv
 *   q = RoPE3D(RMSNorm(q) g_q), k = RoPE3D(RMSNorm(k) g_k) at (frame_pos0 + i / P, row, col)
 *   append k, v to the stream's cache (evicting), then  o = softmax(q K^T / sqrt(128)) V over every
 *   resident token, the chunk's own included;  x += gate1 * (o W_o^T + b_o)
 *   x += softmax(RMSNorm(LN3(x) W_cq^T + b_cq) g_cq K_t^T / sqrt(128)) V_t W_co^T + b_co
 *   x += gate2 * (GELU_tanh((LN(x)(1 + scale2) + shift2) W_1^T + b_1) W_2^T + b_2)
 * x_dev:   fp32 [B, L, C], in place, L = n_frames * tokens_per_frame.
 * e0_dev:  fp32 [B, 6, C].   kt_dev / vtt_dev: this layer's text K/V for each stream of the call, as
 * arrays of B dev pointers held on the host (streams may have different prompts).
 * chunks:  host array [B].  Mutates x and, for each listed stream, this layer's cache and host state.
 * Errors: B < 1 or > SDV2_MAX_BATCH, repeated stream_id, L > W, unequal n_frames, advance = 0
 * without a matching append, workspace smaller than sdv2_block_workspace_bytes(cfg, B, L).
 * ------------------------------------------------------------------------------------------------ */
size_t sdv2_block_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L);
int32_t sdv2_dit_block_forward(const sdv2_model_cfg* cfg, const sdv2_block_weights* w, sdv2_kv_cache* cache,
                               int32_t layer, float* x_dev, const float* e0_dev,
                               const void* const* kt_dev, const void* const* vtt_dev,
                               const sdv2_chunk_desc* chunks, int32_t B,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * One denoising step of a chunk (Section 5.1: 1-4 steps per chunk): conditioning, then blocks
 * 0..n_layers-1 in order, each on its own cache.  Hidden state in, hidden state out.
 * timesteps_host / tvec_dev: as in sdv2_conditioning.
 * kt_dev / vtt_dev: host arrays [n_layers * B] of dev pointers, index layer * B + b.
 * Workspace: sdv2_denoise_workspace_bytes(cfg, B, L).
 * ------------------------------------------------------------------------------------------------ */
size_t sdv2_denoise_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L);
int32_t sdv2_denoise_step(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, sdv2_kv_cache* cache,
                          float* x_dev, const float* timesteps_host, const float* tvec_dev,
                          const void* const* kt_dev, const void* const* vtt_dev,
                          const sdv2_chunk_desc* chunks, int32_t B,
                          void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * The same denoising step, recorded once and replayed (Section 1, "Efficiency objectives": every chunk has a per-frame
 * deadline and jitter counts, so the host's share of a step should be as small and as constant as it can be).
 *
 * sdv2_denoise_graph_create records the launch sequence of sdv2_denoise_step for a fixed set of B streams, chunk
 * length and buffers into a HIP graph.  What changes from step to step (each stream's token ids, RoPE frame index,
 * number of resident keys, timestep) lives in a small descriptor in device memory, `state_dev`
 * (sdv2_denoise_graph_state_bytes() bytes, 256-byte aligned, caller-owned, must outlive the handle), which the
 * kernels read at run time.  Everything else is baked in: cfg, the weight pointers, the cache handle, x_dev
 * (fp32 [B, L, C]: the caller puts each step's input there and finds the output there), the text K/V pointers
 * (host arrays [n_layers * B] as for sdv2_denoise_step), the workspace (sdv2_denoise_workspace_bytes(cfg, B, L)),
 * and the kernel plans, which are those of a full cache.  Recording launches nothing and changes no cache state; it
 * creates one internal stream for the capture.  The graph holds kernel launches only (no memory-set nodes).
 * Errors: as sdv2_denoise_step; per-launch profiling switched on: SDV2_BAD_STATE.
 *
 * sdv2_denoise_graph_launch: one step.  chunks[b] must name the recorded streams in the recorded order with the
 * recorded n_frames; frame_pos0 and advance are free, with the meaning they have in sdv2_denoise_step.  The call
 * validates, enqueues one small kernel that stores the descriptor and then the graph on hip_stream, and advances the
 * host ring state exactly as sdv2_denoise_step does; it does not synchronise.  Steps of one handle must be ordered on
 * one stream.  Results are those of sdv2_denoise_step (bit for bit where the kernel plans coincide, which they do
 * once the cache is full).
 * Errors: a stream whose layers are not in step with each other (the block-level call was used on some of them),
 * advance = 0 without a matching append: SDV2_BAD_STATE, nothing enqueued, state untouched.
 * ------------------------------------------------------------------------------------------------ */
typedef struct sdv2_denoise_graph sdv2_denoise_graph;   /* opaque host handle */
size_t sdv2_denoise_graph_state_bytes(void);
int32_t sdv2_denoise_graph_create(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, sdv2_kv_cache* cache,
                                  float* x_dev, const void* const* kt_dev, const void* const* vtt_dev,
                                  const int32_t* stream_ids, int32_t B, int32_t n_frames,
                                  void* workspace_dev, size_t workspace_bytes, void* state_dev, size_t state_bytes,
                                  sdv2_denoise_graph** out);
int32_t sdv2_denoise_graph_launch(sdv2_denoise_graph* graph, const float* timesteps_host,
                                  const sdv2_chunk_desc* chunks, int32_t B, void* hip_stream);
int32_t sdv2_denoise_graph_destroy(sdv2_denoise_graph* graph);

/* ------------------------------------------------------------------------------------------------
 * Stream batch over denoising steps (Section 1, contribution (1): inputs reformulated as a batch of short chunks;
 * Section 4.2 and its pipeline-parallel stream-batch figure: the n denoising steps of a chunk act as a batch
 * multiplier, L(T, n B), the rows are latent streams at different noise levels, and a clean latent leaves at every
 * micro-step; Section 5.4: more steps, deeper pipeline).
 *
 * The paper prints no schedule; this library takes: a stream denoised in n_steps steps per chunk keeps n_steps chunks
 * in flight.  One micro-step = the newest chunk enters at depth 0, every in-flight chunk makes one denoising step at
 * its depth d with timesteps_host[d], all of them in ONE batched sdv2_denoise_step (n_steps rows in steady state),
 * and the chunk that has finished depth n_steps - 1 leaves.  Each depth has its own rolling cache stream
 * (cache_stream_ids[d], distinct): what a chunk writes at depth d is the history that the following chunks read at
 * depth d.  Chunk c leaves at micro-step c + n_steps - 1.  The rotation is by index: a chunk stays in the row of
 * `rows_dev` it entered until it leaves; only the entering and the leaving chunk are copied ([L, C] fp32 each).
 *
 * sdv2_stream_batch_create: rows_dev = caller-owned fp32 [n_steps][L][C] (256-byte aligned,
 *   sdv2_stream_batch_rows_bytes), L = n_frames * tokens_per_frame.  The cache handle passed to the steps must have
 *   every cache_stream_ids[d] as a stream.  _destroy frees the host handle; _reset empties the pipeline (host only;
 *   resetting the cache streams is the caller's).
 * sdv2_stream_batch_step: x_in_dev = the entering chunk's hidden state (dev fp32 [L, C]) with its RoPE frame index
 *   frame_pos0, or NULL when nothing enters (the pipeline drains: the occupied rows may then form two runs in memory
 *   and the micro-step issues two batched calls).  kt_dev / vtt_dev: host arrays [n_layers] of this stream's text
 *   K/V.  *emitted_out = 1 when a chunk left, its hidden state then being in x_out_dev (dev fp32 [L, C]);
 *   *rows_out (optional) = batch rows of this micro-step.  Workspace: sdv2_denoise_workspace_bytes(cfg, n_steps, L).
 *   Asynchronous on hip_stream like every other call.
 * Errors: as sdv2_denoise_step; n_steps outside 1 .. SDV2_MAX_BATCH, repeated cache stream ids: SDV2_INVALID_ARG.
 *   If a launch fails after part of a micro-step has run, the handle refuses further steps (SDV2_BAD_STATE) until
 *   sdv2_stream_batch_reset.
 * ------------------------------------------------------------------------------------------------ */
typedef struct sdv2_stream_batch sdv2_stream_batch;   /* opaque host handle */
size_t sdv2_stream_batch_rows_bytes(const sdv2_model_cfg* cfg, int32_t n_steps, int32_t n_frames);
int32_t sdv2_stream_batch_create(const sdv2_model_cfg* cfg, int32_t n_steps, const int32_t* cache_stream_ids,
                                 int32_t n_frames, float* rows_dev, size_t rows_bytes, sdv2_stream_batch** out);
int32_t sdv2_stream_batch_destroy(sdv2_stream_batch* sb);
int32_t sdv2_stream_batch_reset(sdv2_stream_batch* sb);
int32_t sdv2_stream_batch_step(sdv2_stream_batch* sb, const sdv2_model_cfg* cfg, const sdv2_model_weights* mw,
                               sdv2_kv_cache* cache, const float* x_in_dev, int32_t frame_pos0,
                               const float* timesteps_host, const void* const* kt_dev, const void* const* vtt_dev,
                               float* x_out_dev, int32_t* emitted_out, int32_t* rows_out,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Latents in, latents out.  The paper runs its causal DiT on VAE latents in 1-4 denoising steps per chunk
 * (Section 5.1), at 2 x 2 latent positions per token (Appendix B: 60 x 104 latent positions -> 1 560 tokens) and gives
 * each incoming chunk a noise rate s_t (Section 4.1, motion-aware noise scheduler); it prints no formula for the
 * steps between latents and the blocks' hidden state, so the ones below are this library's readings:
 *   latents  z: dev fp32 [B][16][F][2 grid_h][2 grid_w]   (16 = SDV2_LATENT_CHANNELS; F = n_frames of the chunk)
 *   patch embedding   token (f, r, c) gathers the 64 numbers z[ch][f][2r + dr][2c + dc], in the order (ch, dr, dc), and
 *                     x = patch W_pe^T + b_pe        (a 3-D convolution with kernel and stride (1, 2, 2)); x fp32 [B, L, C]
 *   output head       v = unpatch( (LN(x)(1 + scale) + shift) W_head^T + b_head ),  (shift, scale) = head_table + tvec[b],
 *                     the 64 numbers of a token going back to where the patch embedding took them from
 *   noise rate        (1 - s) x + s eps for a clean latent x and noise eps
 *   sampler update    the blocks' output read as the velocity eps - x of the interpolation above:  x0 = z - sigma v;
 *                     z_next = x0 when sigma_next = 0, else (1 - sigma_next) x0 + sigma_next eps_next (fresh noise,
 *                     passed in); the timestep fed to the blocks at noise level sigma is 1000 sigma.
 * sdv2_timestep_vector: tvec (dev fp32 [B, C]) of the timesteps, the first line of sdv2_conditioning; workspace
 *   sdv2_conditioning_workspace_bytes.   sdv2_patch_embed / sdv2_output_head: workspace sdv2_latent_io_workspace_bytes.
 * sdv2_noise_latents / sdv2_sampler_update: elementwise over B x elems_per_stream fp32 values with one rate (sigma,
 *   sigma_next) per stream, host arrays [B]; z_next_dev may be z_dev; x0_dev is optional; eps_next_dev may be NULL when
 *   every sigma_next is 0.
 * sdv2_denoise_latents_step: timestep vector, patch embedding, sdv2_denoise_step (with that vector), output head and
 *   sampler update in one call; z_dev is updated in place, chunks / kt_dev / vtt_dev as in sdv2_denoise_step, workspace
 *   sdv2_denoise_latents_workspace_bytes(cfg, B, L).
 * Errors: null pointers, B outside 1 .. SDV2_MAX_BATCH, rates outside [0, 1], sigma_next > sigma: SDV2_INVALID_ARG;
 *   otherwise those of the calls they are made of.
 * ------------------------------------------------------------------------------------------------ */
#define SDV2_LATENT_CHANNELS 16
typedef struct sdv2_io_weights {
    uint32_t struct_size;
    uint32_t reserved;
    const void* W_pe;          /* bf16 [C, 64] */
    const float* b_pe;         /* [C] */
    const float* head_table;   /* [2, C]: shift, scale (added to tvec) */
    const void* W_head;        /* bf16 [64, C] */
    const float* b_head;       /* [64] */
} sdv2_io_weights;
int32_t sdv2_timestep_vector(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, int32_t B,
                             const float* timesteps_host, float* tvec_dev, void* workspace_dev, size_t workspace_bytes,
                             void* hip_stream);
size_t sdv2_latent_io_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L);
int32_t sdv2_patch_embed(const sdv2_model_cfg* cfg, const sdv2_io_weights* io, const float* z_dev, int32_t B,
                         int32_t n_frames, float* x_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream);
int32_t sdv2_output_head(const sdv2_model_cfg* cfg, const sdv2_io_weights* io, const float* x_dev, const float* tvec_dev,
                         int32_t B, int32_t n_frames, float* v_dev, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream);
int32_t sdv2_noise_latents(const float* x_dev, const float* eps_dev, float* out_dev, int32_t B, int64_t elems_per_stream,
                           const float* rate_host, void* hip_stream);
int32_t sdv2_sampler_update(const float* z_dev, const float* v_dev, const float* eps_next_dev, float* z_next_dev,
                            float* x0_dev, int32_t B, int64_t elems_per_stream, const float* sigma_host,
                            const float* sigma_next_host, void* hip_stream);
size_t sdv2_denoise_latents_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L);
int32_t sdv2_denoise_latents_step(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, const sdv2_io_weights* io,
                                  sdv2_kv_cache* cache, float* z_dev, const float* eps_next_dev, float* x0_dev,
                                  const float* sigma_host, const float* sigma_next_host,
                                  const void* const* kt_dev, const void* const* vtt_dev,
                                  const sdv2_chunk_desc* chunks, int32_t B,
                                  void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* The stream batch over denoising steps (Section 4.2) with rows of LATENTS at different noise levels, which is how the
 * paper words it: the rotation of sdv2_stream_batch_step, each micro-step one batched sdv2_denoise_latents_step.
 *   sigmas_host [n_steps + 1]: the noise levels, falling, sigmas_host[d] > 0 for d < n_steps; the row at depth d is
 *     taken from sigmas_host[d] to sigmas_host[d + 1] (timestep 1000 sigmas_host[d]); with sigmas_host[n_steps] = 0
 *     the chunk that leaves is the clean latent.
 *   z_in_dev: the entering chunk's latent at level sigmas_host[0] (dev fp32 [16][F][2 grid_h][2 grid_w]; see
 *     sdv2_noise_latents), or NULL when nothing enters.
 *   eps_by_depth_dev: dev fp32 [n_steps] latents, entry d = the fresh noise for the chunk now at depth d (mixed in at
 *     level sigmas_host[d + 1]; entries whose new level is 0 are not read); NULL allowed when every later level is 0.
 *   z_out_dev: receives the leaving chunk's latent when *emitted_out = 1.
 * The handle is the one of sdv2_stream_batch_create (its rows buffer is large enough for latents); one handle serves
 * one kind of row until sdv2_stream_batch_reset (SDV2_BAD_STATE otherwise).  Workspace:
 * sdv2_stream_batch_latents_workspace_bytes.  Errors as sdv2_stream_batch_step and sdv2_denoise_latents_step. */
size_t sdv2_stream_batch_latents_workspace_bytes(const sdv2_model_cfg* cfg, int32_t n_steps, int32_t n_frames);
int32_t sdv2_stream_batch_latents_step(sdv2_stream_batch* sb, const sdv2_model_cfg* cfg, const sdv2_model_weights* mw,
                                       const sdv2_io_weights* io, sdv2_kv_cache* cache, const float* z_in_dev,
                                       int32_t frame_pos0, const float* sigmas_host, const float* eps_by_depth_dev,
                                       const void* const* kt_dev, const void* const* vtt_dev, float* z_out_dev,
                                       int32_t* emitted_out, int32_t* rows_out,
                                       void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * The two dense kernels on their own (used by the per-kernel parity tests and the benchmark).
 *
 * sdv2_gemm_bf16: out = epilogue(a W^T + bias).  a: bf16 [M, K]; w: bf16 [N, K]; bias fp32 [N] or NULL.
 *   epilogue 0: out bf16 [M, N] = acc + bias
 *            1: out bf16 [M, N] = GELU_tanh(acc + bias)
 *            2: out fp32 [M, N] += gate[row / rows_per_gate][n] * (acc + bias), gate = gate_a[n] +
 *               gate_b[(row / rows_per_gate) * gate_b_stride + n]
 *            3: out fp32 [M, N] += acc + bias
 *   K multiple of 64, N multiple of 128 (else SDV2_INVALID_ARG).
 *   workspace_dev (device, 16-byte aligned; may be NULL with workspace_bytes 0): scratch that lets a shape with few
 *   output tiles and a long k split the k range over several workgroups per tile (a second small kernel adds the parts in
 *   k order, so the result does not depend on scheduling).  A workspace smaller than
 *   sdv2_gemm_workspace_bytes(M, N, K, epilogue) is accepted: the launch then does not split.
 *
 * sdv2_attention_bf16: o[b] = softmax(q[b] K[b]^T / sqrt(128)) V[b] over kv_len[b] slots.
 *   q: bf16 [B, L, C]; k[b]: bf16 [H][cap][128]; vt[b]: bf16 [H][128][cap] in the cache's column order (cap multiple of 64,
 *   >= kv_len[b] > 0); o: bf16 [B, L, C].  workspace: sdv2_attention_workspace_bytes(B, L, C, max kv_len).
 * ------------------------------------------------------------------------------------------------ */
size_t sdv2_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t epilogue);
int32_t sdv2_gemm_bf16(const void* a_dev, const void* w_dev, const float* bias_dev, void* out_dev,
                       int32_t M, int32_t N, int32_t K, int32_t epilogue,
                       const float* gate_a_dev, const float* gate_b_dev, int32_t gate_b_stride,
                       int32_t rows_per_gate, void* workspace_dev, size_t workspace_bytes, void* hip_stream);
/* sdv2_gemm_bf16_noalloc: sdv2_gemm_bf16 for callers that cannot allocate device memory and have no workspace to
 * hand over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments,
 * layouts, epilogues and results as sdv2_gemm_bf16 called with a full workspace; the k-split's fp32 partial sums go
 * to a scratch array built into the library's device image (sdv2_gemm_noalloc_max_scratch_bytes() = 32 MiB per GPU
 * that loads the library, held until the process ends).  The call allocates nothing, frees nothing, and does not
 * synchronise.
 * Errors: a shape whose planned k-split needs more than that scratch: SDV2_INVALID_ARG (use sdv2_gemm_bf16 with a
 * workspace); otherwise as sdv2_gemm_bf16.
 * Every call on one GPU uses that GPU's one scratch array: calls that overlap in time on the same GPU (different
 * streams) race on it; calls ordered on one stream do not.  Nothing in the scratch has to start at zero: every
 * partial sum that the reduce pass reads is stored by the same call first. */
size_t sdv2_gemm_noalloc_max_scratch_bytes(void);
int32_t sdv2_gemm_bf16_noalloc(const void* a_dev, const void* w_dev, const float* bias_dev, void* out_dev,
                               int32_t M, int32_t N, int32_t K, int32_t epilogue,
                               const float* gate_a_dev, const float* gate_b_dev, int32_t gate_b_stride,
                               int32_t rows_per_gate, void* hip_stream);
size_t sdv2_attention_workspace_bytes(int32_t B, int32_t L, int32_t C, int32_t max_kv_len);
int32_t sdv2_attention_bf16(const void* q_dev, const void* const* k_dev, const void* const* vt_dev,
                            const int32_t* kv_len_host, const int32_t* cap_host, void* o_dev,
                            int32_t B, int32_t L, int32_t n_heads,
                            void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Per-launch timing for the benchmark (not part of the streaming path).  Between sdv2_prof_begin and
 * sdv2_prof_end every kernel launch site of sdv2_dit_block_forward / sdv2_denoise_step is bracketed by
 * a pair of HIP events on the caller's stream, up to max_samples launches.  sdv2_prof_end waits for
 * the recorded events (the only call of the library that blocks), writes one (tag, milliseconds) per
 * launch in launch order into the host arrays and destroys the events.  Not thread safe.
 * ------------------------------------------------------------------------------------------------ */
enum sdv2_launch_tag {
    SDV2_TAG_ADALN1 = 0, SDV2_TAG_QKV = 1, SDV2_TAG_ROPE_APPEND = 2, SDV2_TAG_SELF_ATTN = 3,
    SDV2_TAG_OUT_PROJ = 4, SDV2_TAG_LN3 = 5, SDV2_TAG_CROSS_Q = 6, SDV2_TAG_CROSS_Q_NORM = 7,
    SDV2_TAG_CROSS_ATTN = 8, SDV2_TAG_CROSS_OUT = 9, SDV2_TAG_ADALN2 = 10, SDV2_TAG_FFN1 = 11,
    SDV2_TAG_FFN2 = 12,
    SDV2_TAG_GEMM_REDUCE = 13,    /* second pass of a product whose k range was split: sum of the parts + epilogue
                                     (+ the next LayerNorm when it is fused in) */
    SDV2_TAG_ATTN_MERGE = 14,     /* second pass of an attention whose key range was split over workgroups */
    SDV2_TAG_COUNT = 15
};
int32_t sdv2_prof_begin(int32_t max_samples);
int32_t sdv2_prof_end(int32_t* tags_out, float* ms_out, int32_t capacity, int32_t* n_out);

/* ------------------------------------------------------------------------------------------------
 * What the chip sustains, measured by the benchmark beside the published peaks (not part of the streaming path).
 * sdv2_prof_peak_mfma: `workgroups` workgroups of eight waves, each wave issuing iters x 8 independent
 *   v_mfma_f32_32x32x16_bf16 on register operands (no memory traffic); *flops_out = the flops of the launch
 *   (2 x 32 x 32 x 16 per instruction).  sink_dev: dev fp32 [workgroups * 512], written once at the end.
 * sdv2_prof_peak_copy: dst <- src, `bytes` (multiple of 16) bytes, 16-byte accesses, grid-stride; moves 2 x bytes
 *   through HBM when the buffers exceed the caches.
 * Both only enqueue one kernel; the caller times it with events on the same stream.
 * sdv2_prof_lds_rates: three launches of one workgroup of eight waves, each wave issuing iters x 8 times the same LDS
 *   instruction of 16 bytes per lane (1 KB per wave instruction): ds_read_b128, ds_write_b128, and the direct
 *   global -> LDS load; the shader clocks each took (s_memtime, first instruction to last result) are left as three
 *   uint64 at the start of scratch_dev (dev, 256-byte aligned, >= 40960 bytes, contents overwritten; the direct loads
 *   read its bytes 8192 .. 40959).  Clocks per wave instruction = ticks / (iters * 8 * 8).  Enqueue only.
 * ------------------------------------------------------------------------------------------------ */
/* sdv2_prof_kernel_name: the kernel instantiation the library's planner picks, spelled as a profiler prints it, so
 * that the benchmark can group launch sites by kernel the way a rocprofv3 summary does.
 *   kind 0: the GEMM of B * L rows with N = a0, K = a1, epilogue a2;  kind 1: attention of B streams x L queries,
 *   a0 heads, a1 keys, cache capacity a2 slots.  Host only; `out` receives a NUL-terminated string. */
int32_t sdv2_prof_kernel_name(int32_t kind, int32_t B, int32_t L, int32_t a0, int32_t a1, int32_t a2, char* out,
                              size_t capacity);
int32_t sdv2_prof_peak_mfma(int32_t iters, int32_t workgroups, float* sink_dev, size_t sink_floats, double* flops_out,
                            void* hip_stream);
int32_t sdv2_prof_peak_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream);
int32_t sdv2_prof_lds_rates(int32_t iters, void* scratch_dev, size_t scratch_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Tuning hook for tests and sweeps (not for production use, not thread safe): replaces the library's own choice of
 * a kernel plan until cleared with value NULL or "".  It changes workspace sizes too, so set it before the
 * *_workspace_bytes query that goes with a call.  Nothing is read from the environment.
 *   "gemm_tile":   "tm,tn[,pf[,k_parts]]" (register-staged kernel, tile 128 tm x 32 tn) or "d<id>[,k_parts]"
 *                  (a configuration of the direct-to-LDS kernel)
 *   "attn_waves":  "4" or "8": query blocks (waves) per attention workgroup, one key stream; "2": the key-split form
 *                  (2 query blocks x 4 key slices per workgroup; used only when every capacity is a multiple of 128)
 *   "attn_splits": parts of the key range over workgroups (1 .. 16)
 * Errors: unknown name or a value that does not parse: SDV2_INVALID_ARG (the previous setting stays).
 * ------------------------------------------------------------------------------------------------ */
int32_t sdv2_tuning_set(const char* name, const char* value);

#ifdef __cplusplus
}
#endif
#endif /* SDV2_H */
