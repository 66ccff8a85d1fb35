// Host side of libsdv2: argument validation, ring bookkeeping, workspace carving and the launch
// sequence of the block.  See include/sdv2.h for the contract of every exported call.
#include "common.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/sdv2.h"

using namespace sdv2;

// ------------------------------------------------------------------------------------------ errors
namespace {

thread_local std::string g_last_error;

int32_t fail(int32_t code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

int32_t hip_fail(hipError_t e, const char* what) {
    return fail(SDV2_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(expr, what)                           \
    do {                                              \
        hipError_t e__ = (expr);                      \
        if (e__ != hipSuccess) return hip_fail(e__, what); \
    } while (0)

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Optional per-launch timing with HIP events (sdv2_prof_begin / sdv2_prof_end).
struct Profiler {
    bool on = false;
    int n = 0;
    std::vector<hipEvent_t> start, stop;
    std::vector<int> tag;
};
Profiler g_prof;

template <typename F>
hipError_t timed(int tag, hipStream_t s, F&& launch) {
    if (!g_prof.on || g_prof.n >= (int)g_prof.start.size()) return launch();
    const int i = g_prof.n++;
    g_prof.tag[i] = tag;
    hipError_t e = hipEventRecord(g_prof.start[i], s);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    return hipEventRecord(g_prof.stop[i], s);
}

bool model_cfg_ok(const sdv2_model_cfg* c, const char** why) {
    *why = nullptr;
    if (!c) *why = "cfg is null";
    else if (c->struct_size != sizeof(sdv2_model_cfg)) *why = "cfg.struct_size mismatch";
    else if (c->n_heads <= 0 || c->C != c->n_heads * SDV2_HEAD_DIM) *why = "C must equal n_heads * 128";
    else if (c->C > 8192) *why = "C > 8192";
    else if (c->ffn_dim <= 0 || c->ffn_dim % 128) *why = "ffn_dim must be a positive multiple of 128";
    else if (c->grid_h <= 0 || c->grid_w <= 0) *why = "grid must be positive";
    else if (c->text_len <= 0) *why = "text_len must be positive";
    else if (c->n_layers <= 0) *why = "n_layers must be positive";
    else if (c->t_dim <= 0 || c->t_dim % 8) *why = "t_dim must be a positive multiple of 8";
    else if (!(c->eps > 0.0f) || !(c->rope_base > 1.0f)) *why = "eps / rope_base out of range";
    return *why == nullptr;
}

}  // namespace

// ------------------------------------------------------------------------------------------ cache handle
struct sdv2_kv_cache {
    sdv2_cache_cfg cfg;
    int cap;                       // S + W rounded up to 64
    unsigned char* base;
    size_t k_bytes, ids_bytes, unit_bytes;   // per (layer, stream)
    std::vector<int64_t> total;    // [layer * n_streams + stream]
    std::vector<int32_t> last_n;   // size of the most recent advancing append (0: none); negated once a sink
                                   // refresh has closed that chunk (advance = 0 is then refused)
    std::vector<std::vector<int64_t>> sink_ids;   // per (layer, stream): ids held by the sink slots after a
                                                  // refresh (empty: the first S tokens, the closed form)
};

namespace {

bool cache_cfg_ok(const sdv2_cache_cfg* c, const char** why) {
    *why = nullptr;
    if (!c) *why = "cfg is null";
    else if (c->struct_size != sizeof(sdv2_cache_cfg)) *why = "cfg.struct_size mismatch";
    else if (c->n_layers <= 0 || c->n_streams <= 0 || c->n_heads <= 0) *why = "n_layers, n_streams, n_heads must be positive";
    else if (c->tokens_per_frame <= 0) *why = "tokens_per_frame must be positive";
    else if (c->sink_tokens < 0) *why = "sink_tokens < 0";
    else if (c->window_tokens <= 0) *why = "window_tokens <= 0";
    else if (c->sink_tokens % c->tokens_per_frame || c->window_tokens % c->tokens_per_frame)
        *why = "sink_tokens and window_tokens must be whole frames";
    else if ((int64_t)c->sink_tokens + c->window_tokens > (1 << 30)) *why = "cache too large";
    return *why == nullptr;
}

void cache_geometry(const sdv2_cache_cfg* c, int* cap, size_t* k_bytes, size_t* ids_bytes, size_t* unit) {
    *cap = (int)align_up((size_t)c->sink_tokens + c->window_tokens, 64);
    *k_bytes = (size_t)c->n_heads * *cap * SDV2_HEAD_DIM * sizeof(bf16);
    *ids_bytes = (size_t)*cap * sizeof(int64_t);
    *unit = align_up(2 * *k_bytes + *ids_bytes, 256);
}

int slot_of_host(int64_t g, int S, int W) { return g < S ? (int)g : S + (int)((g - S) % W); }

int32_t check_layer_stream(const sdv2_kv_cache* c, int32_t layer, int32_t stream) {
    if (!c) return fail(SDV2_INVALID_ARG, "cache handle is null");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(SDV2_INVALID_ARG, "layer %d out of range", layer);
    if (stream < 0 || stream >= c->cfg.n_streams) return fail(SDV2_INVALID_ARG, "stream %d out of range", stream);
    return SDV2_OK;
}

AppendStream append_stream(const sdv2_kv_cache* c, int layer, int stream, int64_t g0, int frame_pos0) {
    unsigned char* u = c->base + ((size_t)layer * c->cfg.n_streams + stream) * c->unit_bytes;
    AppendStream s;
    s.k_cache = reinterpret_cast<bf16*>(u);
    s.vt_cache = reinterpret_cast<bf16*>(u + c->k_bytes);
    s.ids = reinterpret_cast<long long*>(u + 2 * c->k_bytes);
    s.g0 = g0;
    s.frame_pos0 = frame_pos0;
    s.cap = c->cap;
    return s;
}

}  // namespace

extern "C" {

const char* sdv2_last_error(void) { return g_last_error.c_str(); }
int32_t sdv2_version(void) { return 2; }

int32_t sdv2_tuning_set(const char* name, const char* value) {
    if (!name) return fail(SDV2_INVALID_ARG, "name is null");
    const bool clear = !value || !*value;
    if (!strcmp(name, "gemm_tile")) {
        if (!set_gemm_tile_override(clear ? nullptr : value)) return fail(SDV2_INVALID_ARG, "gemm_tile \"%s\" not understood", value);
        return SDV2_OK;
    }
    if (!strcmp(name, "attn_waves") || !strcmp(name, "attn_splits")) {
        const int v = clear ? 0 : atoi(value);
        if (v < 0) return fail(SDV2_INVALID_ARG, "%s must be >= 0", name);
        if (!strcmp(name, "attn_waves")) {
            if (v != 0 && v != 2 && v != 4 && v != 8) return fail(SDV2_INVALID_ARG, "attn_waves must be 0, 2, 4 or 8");
            set_attention_overrides(v, -1);
        } else {
            set_attention_overrides(-1, v);
        }
        return SDV2_OK;
    }
    return fail(SDV2_INVALID_ARG, "unknown tuning name \"%s\"", name);
}

size_t sdv2_kv_cache_bytes(const sdv2_cache_cfg* cfg) {
    const char* why;
    if (!cache_cfg_ok(cfg, &why)) {
        fail(SDV2_INVALID_ARG, "%s", why);
        return 0;
    }
    int cap;
    size_t kb, ib, unit;
    cache_geometry(cfg, &cap, &kb, &ib, &unit);
    return unit * cfg->n_layers * cfg->n_streams;
}

int32_t sdv2_kv_cache_init(const sdv2_cache_cfg* cfg, void* dev_storage, size_t bytes, sdv2_kv_cache** out) {
    const char* why;
    if (!cache_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!dev_storage || !out) return fail(SDV2_INVALID_ARG, "null pointer");
    if (reinterpret_cast<uintptr_t>(dev_storage) % 256) return fail(SDV2_INVALID_ARG, "storage must be 256-byte aligned");
    const size_t need = sdv2_kv_cache_bytes(cfg);
    if (bytes < need) return fail(SDV2_INVALID_ARG, "storage too small: %zu < %zu", bytes, need);
    sdv2_kv_cache* c = new (std::nothrow) sdv2_kv_cache;
    if (!c) return fail(SDV2_INVALID_ARG, "out of host memory");
    c->cfg = *cfg;
    cache_geometry(cfg, &c->cap, &c->k_bytes, &c->ids_bytes, &c->unit_bytes);
    c->base = static_cast<unsigned char*>(dev_storage);
    c->total.assign((size_t)cfg->n_layers * cfg->n_streams, 0);
    c->last_n.assign((size_t)cfg->n_layers * cfg->n_streams, 0);
    c->sink_ids.assign((size_t)cfg->n_layers * cfg->n_streams, std::vector<int64_t>());
    *out = c;
    return SDV2_OK;
}

int32_t sdv2_kv_cache_destroy(sdv2_kv_cache* cache) {
    delete cache;
    return SDV2_OK;
}

int32_t sdv2_kv_cache_reset(sdv2_kv_cache* cache, int32_t stream_id) {
    int32_t rc = check_layer_stream(cache, 0, stream_id);
    if (rc) return rc;
    for (int l = 0; l < cache->cfg.n_layers; ++l) {
        cache->total[(size_t)l * cache->cfg.n_streams + stream_id] = 0;
        cache->last_n[(size_t)l * cache->cfg.n_streams + stream_id] = 0;
        cache->sink_ids[(size_t)l * cache->cfg.n_streams + stream_id].clear();
    }
    return SDV2_OK;
}

int32_t sdv2_kv_cache_state(const sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, sdv2_cache_state* out) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    if (!out) return fail(SDV2_INVALID_ARG, "out is null");
    const int S = cache->cfg.sink_tokens, W = cache->cfg.window_tokens;
    const int64_t total = cache->total[(size_t)layer * cache->cfg.n_streams + stream_id];
    out->total = total;
    out->sink_fill = (int32_t)(total < S ? total : S);
    const int64_t in_win = total > S ? total - S : 0;
    out->win_fill = (int32_t)(in_win < W ? in_win : W);
    out->evicted = in_win > W ? in_win - W : 0;
    out->oldest_slot = out->win_fill ? slot_of_host(total - out->win_fill, S, W) : -1;
    out->next_slot = slot_of_host(total, S, W);
    return SDV2_OK;
}

int32_t sdv2_kv_cache_slot_map(const sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int64_t* slot_map_out) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    if (!slot_map_out) return fail(SDV2_INVALID_ARG, "slot_map_out is null");
    const int S = cache->cfg.sink_tokens, W = cache->cfg.window_tokens;
    const int64_t total = cache->total[(size_t)layer * cache->cfg.n_streams + stream_id];
    for (int i = 0; i < S + W; ++i) slot_map_out[i] = -1;
    const int64_t sink_end = total < S ? total : S;
    const std::vector<int64_t>& refreshed = cache->sink_ids[(size_t)layer * cache->cfg.n_streams + stream_id];
    for (int64_t g = 0; g < sink_end; ++g) slot_map_out[g] = refreshed.empty() ? g : refreshed[(size_t)g];
    int64_t first = total - W;
    if (first < S) first = S;
    for (int64_t g = first; g < total; ++g) slot_map_out[slot_of_host(g, S, W)] = g;
    return SDV2_OK;
}

int32_t sdv2_kv_cache_device_ptrs(const sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, void** k_dev,
                                  void** vt_dev, int64_t** ids_dev, int32_t* cap) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    AppendStream s = append_stream(cache, layer, stream_id, 0, 0);
    if (k_dev) *k_dev = s.k_cache;
    if (vt_dev) *vt_dev = s.vt_cache;
    if (ids_dev) *ids_dev = reinterpret_cast<int64_t*>(s.ids);
    if (cap) *cap = cache->cap;
    return SDV2_OK;
}

int32_t sdv2_kv_cache_append_evict(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, const void* k_dev,
                                   const void* v_dev, int32_t n_tokens, int32_t advance, void* hip_stream) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    if (!k_dev || !v_dev) return fail(SDV2_INVALID_ARG, "k/v is null");
    const sdv2_cache_cfg& cf = cache->cfg;
    if (n_tokens <= 0 || n_tokens > cf.window_tokens || n_tokens % cf.tokens_per_frame)
        return fail(SDV2_INVALID_ARG, "n_tokens %d must be whole frames, positive and at most the window", n_tokens);
    const size_t idx = (size_t)layer * cf.n_streams + stream_id;
    if (!advance && cache->last_n[idx] != n_tokens)
        return fail(SDV2_BAD_STATE, "advance = 0 needs a previous append of %d tokens (last was %d)", n_tokens,
                    cache->last_n[idx]);
    const int64_t old_total = cache->total[idx];
    const int32_t old_last = cache->last_n[idx];
    if (advance) {
        cache->total[idx] += n_tokens;
        cache->last_n[idx] = n_tokens;
    }
    PlainAppendArgs a;
    a.k = static_cast<const bf16*>(k_dev);
    a.v = static_cast<const bf16*>(v_dev);
    a.n = n_tokens;
    a.C = cf.n_heads * SDV2_HEAD_DIM;
    a.H = cf.n_heads;
    a.S = cf.sink_tokens;
    a.W = cf.window_tokens;
    a.st = append_stream(cache, layer, stream_id, cache->total[idx] - n_tokens, 0);
    hipError_t e = launch_plain_append(a, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        cache->total[idx] = old_total;
        cache->last_n[idx] = old_last;
        return hip_fail(e, "append kernel");
    }
    return SDV2_OK;
}

// ------------------------------------------------------------------------------------------ sink / RoPE refresh
namespace {
// First slot of frame `frame_back` (0 = last) of the most recent append; < 0 with an error set.
int32_t latest_frame_slot(const sdv2_kv_cache* cache, size_t idx, int32_t frame_back, int* slot0) {
    const sdv2_cache_cfg& cf = cache->cfg;
    const int P = cf.tokens_per_frame;
    const int last = cache->last_n[idx] < 0 ? -cache->last_n[idx] : cache->last_n[idx];
    if (last == 0) return fail(SDV2_BAD_STATE, "nothing has been appended yet");
    if (frame_back < 0 || frame_back >= last / P)
        return fail(SDV2_INVALID_ARG, "frame_back %d outside the latest append of %d frames", frame_back, last / P);
    const int64_t g0 = cache->total[idx] - (int64_t)(frame_back + 1) * P;
    if (g0 < cf.sink_tokens) return fail(SDV2_BAD_STATE, "that frame was stored in the sink itself");
    *slot0 = slot_of_host(g0, cf.sink_tokens, cf.window_tokens);
    return SDV2_OK;
}
}  // namespace

size_t sdv2_sink_similarity_workspace_bytes(const sdv2_kv_cache* cache) {
    if (!cache) return 0;
    const int m = cache->cfg.sink_tokens / cache->cfg.tokens_per_frame;
    return align_up((size_t)(m > 0 ? m : 1) * sink_similarity_blocks(cache->cfg.n_heads) * 3 * sizeof(float), 256);
}

int32_t sdv2_sink_similarity(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int32_t frame_back,
                             float* alpha_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    if (!alpha_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "alpha / workspace is null");
    const sdv2_cache_cfg& cf = cache->cfg;
    const size_t idx = (size_t)layer * cf.n_streams + stream_id;
    const int m = cf.sink_tokens / cf.tokens_per_frame;
    if (m == 0) return fail(SDV2_BAD_STATE, "the cache has no sink");
    if (cache->total[idx] < cf.sink_tokens) return fail(SDV2_BAD_STATE, "the sink is not filled yet");
    if (workspace_bytes < sdv2_sink_similarity_workspace_bytes(cache))
        return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes,
                    sdv2_sink_similarity_workspace_bytes(cache));
    int src0 = 0;
    rc = latest_frame_slot(cache, idx, frame_back, &src0);
    if (rc) return rc;
    AppendStream st = append_stream(cache, layer, stream_id, 0, 0);
    SinkSimArgs a;
    a.vt = st.vt_cache;
    a.H = cf.n_heads;
    a.cap = cache->cap;
    a.P = cf.tokens_per_frame;
    a.src0 = src0;
    a.m = m;
    a.partial = static_cast<float*>(workspace_dev);
    a.alpha = alpha_dev;
    hipError_t e = launch_sink_similarity(a, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "sink similarity kernel");
    return SDV2_OK;
}

int32_t sdv2_kv_cache_refresh_sink(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int32_t sink_frame,
                                   int32_t frame_back, void* hip_stream) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    const sdv2_cache_cfg& cf = cache->cfg;
    const size_t idx = (size_t)layer * cf.n_streams + stream_id;
    const int P = cf.tokens_per_frame;
    const int m = cf.sink_tokens / P;
    if (sink_frame < 0 || sink_frame >= m) return fail(SDV2_INVALID_ARG, "sink_frame %d out of range (%d sink frames)", sink_frame, m);
    if (cache->total[idx] < cf.sink_tokens) return fail(SDV2_BAD_STATE, "the sink is not filled yet");
    int src0 = 0;
    rc = latest_frame_slot(cache, idx, frame_back, &src0);
    if (rc) return rc;
    AppendStream st = append_stream(cache, layer, stream_id, 0, 0);
    SinkCopyArgs a;
    a.k = st.k_cache;
    a.vt = st.vt_cache;
    a.ids = st.ids;
    a.H = cf.n_heads;
    a.cap = cache->cap;
    a.P = P;
    a.src0 = src0;
    a.dst0 = sink_frame * P;
    hipError_t e = launch_refresh_sink(a, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "sink refresh kernel");
    std::vector<int64_t>& ids = cache->sink_ids[idx];
    if (ids.empty()) {
        ids.resize((size_t)cf.sink_tokens);
        for (int g = 0; g < cf.sink_tokens; ++g) ids[(size_t)g] = g;
    }
    const int64_t g0 = cache->total[idx] - (int64_t)(frame_back + 1) * P;
    for (int j = 0; j < P; ++j) ids[(size_t)sink_frame * P + j] = g0 + j;
    if (cache->last_n[idx] > 0) cache->last_n[idx] = -cache->last_n[idx];      // the chunk is closed
    return SDV2_OK;
}

int32_t sdv2_kv_cache_rotate_keys(sdv2_kv_cache* cache, int32_t layer, int32_t stream_id, int32_t delta_frames,
                                  float rope_base, void* hip_stream) {
    int32_t rc = check_layer_stream(cache, layer, stream_id);
    if (rc) return rc;
    if (!(rope_base > 1.0f)) return fail(SDV2_INVALID_ARG, "rope_base out of range");
    const sdv2_cache_cfg& cf = cache->cfg;
    sdv2_cache_state stt;
    rc = sdv2_kv_cache_state(cache, layer, stream_id, &stt);
    if (rc) return rc;
    AppendStream st = append_stream(cache, layer, stream_id, 0, 0);
    RotateKeysArgs a;
    a.k = st.k_cache;
    a.H = cf.n_heads;
    a.cap = cache->cap;
    a.S = cf.sink_tokens;
    a.sink_fill = stt.sink_fill;
    a.n_slots = stt.sink_fill + stt.win_fill;
    const int pairs = SDV2_HEAD_DIM / 2;
    a.n_pairs = pairs - 2 * (pairs / 3);                          // the frame axis owns the leading pairs
    for (int j = 0; j < kMaxFramePairs; ++j) {
        const double ang = j < a.n_pairs ? -(double)delta_frames * pow((double)rope_base, -(double)j / a.n_pairs) : 0.0;
        a.cs[j] = (float)cos(ang);
        a.sn[j] = (float)sin(ang);
    }
    hipError_t e = launch_rotate_keys(a, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "key rotation kernel");
    return SDV2_OK;
}

// ------------------------------------------------------------------------------------------ motion-aware noise scheduler
namespace {
bool motion_cfg_ok(const sdv2_motion_cfg* c, const char** why) {
    *why = nullptr;
    if (!c) *why = "cfg is null";
    else if (c->struct_size != sizeof(sdv2_motion_cfg)) *why = "cfg.struct_size mismatch";
    else if (c->k < 0 || c->k > kMotionMaxK) *why = "k out of range";
    else if (!(c->sigma > 0.0f)) *why = "sigma must be positive";
    else if (!(c->lambda > 0.0f && c->lambda < 1.0f)) *why = "lambda must lie strictly between 0 and 1";
    else if (!(c->s_min <= c->s_max)) *why = "s_min > s_max";
    return *why == nullptr;
}
size_t motion_ring_floats(const sdv2_motion_cfg* c) { return align_up((size_t)c->k + 1, 16); }
}  // namespace

size_t sdv2_motion_state_bytes(const sdv2_motion_cfg* cfg) {
    const char* why;
    if (!motion_cfg_ok(cfg, &why)) return 0;
    return align_up((kMotionHeaderFloats + motion_ring_floats(cfg) + (size_t)kMotionMaxFrames * kMotionBlocks) * sizeof(float), 256);
}

int32_t sdv2_motion_init(const sdv2_motion_cfg* cfg, void* state_dev, size_t state_bytes, void* hip_stream) {
    const char* why;
    if (!motion_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!state_dev || reinterpret_cast<uintptr_t>(state_dev) % 16) return fail(SDV2_INVALID_ARG, "state is null or not 16-byte aligned");
    const size_t need = sdv2_motion_state_bytes(cfg);
    if (state_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "state %zu < %zu", state_bytes, need);
    hipError_t e = launch_motion_init(static_cast<float*>(state_dev), (int)(need / sizeof(float)), cfg->s_init,
                                      static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "motion init kernel");
    return SDV2_OK;
}

int32_t sdv2_motion_update(const sdv2_motion_cfg* cfg, void* state_dev, size_t state_bytes, const float* frames_dev,
                           const float* prev_frame_dev, int32_t n_frames, int64_t frame_elems, float* d_out_dev,
                           float* dhat_out_dev, float* s_out_dev, void* hip_stream) {
    const char* why;
    if (!motion_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!state_dev || !frames_dev || !d_out_dev || !dhat_out_dev || !s_out_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    if (state_bytes < sdv2_motion_state_bytes(cfg)) return fail(SDV2_WORKSPACE_TOO_SMALL, "state too small");
    if (n_frames <= 0 || n_frames > kMotionMaxFrames) return fail(SDV2_INVALID_ARG, "n_frames %d outside 1 .. %d", n_frames, kMotionMaxFrames);
    if (frame_elems <= 0) return fail(SDV2_INVALID_ARG, "frame_elems must be positive");
    MotionArgs a;
    a.frames = frames_dev;
    a.prev = prev_frame_dev;
    a.n = frame_elems;
    a.T = n_frames;
    a.k = cfg->k;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(frames_dev) | reinterpret_cast<uintptr_t>(prev_frame_dev);
    a.vec4 = (frame_elems % 4 == 0 && bits % 16 == 0) ? 1 : 0;
    a.sigma = cfg->sigma;
    a.lambda = cfg->lambda;
    a.s_min = cfg->s_min;
    a.s_max = cfg->s_max;
    a.state = static_cast<float*>(state_dev);
    a.partial = a.state + kMotionHeaderFloats + motion_ring_floats(cfg);
    a.d_out = d_out_dev;
    a.dhat_out = dhat_out_dev;
    a.s_out = s_out_dev;
    hipError_t e = launch_motion_update(a, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "motion kernels");
    return SDV2_OK;
}

// ------------------------------------------------------------------------------------------ SLO-aware batching scheduler
int32_t sdv2_slo_pick_batch(const int32_t* batch_sizes, const double* latency_s, int32_t n, int32_t frames_per_chunk,
                            double f_slo, int64_t frames_collected, double knee_tol, int32_t* batch_out,
                            double* frequency_out, int32_t* meets_slo_out) {
    if (!batch_sizes || !latency_s || !batch_out) return fail(SDV2_INVALID_ARG, "null pointer");
    if (n <= 0 || frames_per_chunk <= 0) return fail(SDV2_INVALID_ARG, "n and frames_per_chunk must be positive");
    if (!(knee_tol >= 0.0 && knee_tol < 1.0)) return fail(SDV2_INVALID_ARG, "knee_tol must lie in [0, 1)");
    for (int i = 0; i < n; ++i)
        if (batch_sizes[i] < 1 || !(latency_s[i] > 0.0))
            return fail(SDV2_INVALID_ARG, "entry %d: batch size must be >= 1 and latency positive", i);
    // f = B T / L(T, B) of the allowed sizes (B T <= frames collected)
    int best_any = -1, best_ok = -1;
    double f_any = 0.0, f_ok = 0.0;
    auto freq = [&](int i) { return (double)batch_sizes[i] * frames_per_chunk / latency_s[i]; };
    auto allowed = [&](int i) { return (int64_t)batch_sizes[i] * frames_per_chunk <= frames_collected; };
    for (int i = 0; i < n; ++i) {
        if (!allowed(i)) continue;
        const double f = freq(i);
        if (best_any < 0 || f > f_any || (f == f_any && batch_sizes[i] < batch_sizes[best_any])) {
            best_any = i;
            f_any = f;
        }
        if (f >= f_slo && (best_ok < 0 || f > f_ok)) {
            best_ok = i;
            f_ok = f;
        }
    }
    int pick = -1, meets = 0;
    if (best_ok >= 0) {
        // the smallest allowed size that meets the SLO and is within knee_tol of the best such frequency
        for (int i = 0; i < n; ++i) {
            if (!allowed(i)) continue;
            const double f = freq(i);
            if (f >= f_slo && f >= (1.0 - knee_tol) * f_ok && (pick < 0 || batch_sizes[i] < batch_sizes[pick])) pick = i;
        }
        meets = 1;
    } else {
        pick = best_any;
    }
    *batch_out = pick < 0 ? 0 : batch_sizes[pick];
    if (frequency_out) *frequency_out = pick < 0 ? 0.0 : freq(pick);
    if (meets_slo_out) *meets_slo_out = meets;
    return SDV2_OK;
}

// ------------------------------------------------------------------------------------------ dense helpers
size_t sdv2_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K, int32_t epilogue) {
    if (M <= 0 || N <= 0 || K <= 0 || epilogue < 0 || epilogue > 3) return 0;
    return align_up(gemm_splitk_floats(M, N, K, epilogue) * sizeof(float), 256);
}

int32_t sdv2_gemm_bf16(const void* a_dev, const void* w_dev, const float* bias_dev, void* out_dev, int32_t M,
                       int32_t N, int32_t K, int32_t epilogue, const float* gate_a_dev, const float* gate_b_dev,
                       int32_t gate_b_stride, int32_t rows_per_gate, void* workspace_dev, size_t workspace_bytes,
                       void* hip_stream) {
    if (!a_dev || !w_dev || !out_dev) return fail(SDV2_INVALID_ARG, "null operand");
    if (M <= 0 || N <= 0 || K <= 0) return fail(SDV2_INVALID_ARG, "M, N, K must be positive");
    if (K % 64) return fail(SDV2_INVALID_ARG, "K = %d must be a multiple of 64", K);
    if (N % 128) return fail(SDV2_INVALID_ARG, "N = %d must be a multiple of 128", N);
    if (epilogue < 0 || epilogue > 3) return fail(SDV2_INVALID_ARG, "epilogue %d unknown", epilogue);
    if (epilogue == kEpiGatedResidual && (!gate_a_dev || !gate_b_dev || rows_per_gate <= 0))
        return fail(SDV2_INVALID_ARG, "gated epilogue needs gate_a, gate_b and rows_per_gate > 0");
    GemmArgs g;
    g.a = static_cast<const bf16*>(a_dev);
    g.w = static_cast<const bf16*>(w_dev);
    g.bias = bias_dev;
    g.out = out_dev;
    g.M = M;
    g.N = N;
    g.K = K;
    g.epilogue = epilogue;
    g.gate_a = gate_a_dev;
    g.gate_b = gate_b_dev;
    g.gate_b_stride = gate_b_stride;
    g.rows_per_gate = rows_per_gate > 0 ? rows_per_gate : 1;
    g.splitk_partials = nullptr;
    g.splitk_floats = 0;
    if (workspace_dev && workspace_bytes) {
        if (reinterpret_cast<uintptr_t>(workspace_dev) % 16) return fail(SDV2_INVALID_ARG, "workspace must be 16-byte aligned");
        g.splitk_partials = static_cast<float*>(workspace_dev);
        g.splitk_floats = workspace_bytes / sizeof(float);
    }
    HIP_TRY(launch_gemm(g, static_cast<hipStream_t>(hip_stream)), "gemm kernel");
    return SDV2_OK;
}

// ---- the same product for callers that cannot allocate: the k-split scratch lives in the library's image
}  // extern "C"

namespace {
constexpr size_t kNoAllocScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
// One copy per GPU that loads the library, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress: the device address differs per GPU and is looked up once per device below.
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call on that device).
int32_t noalloc_scratch(void** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(SDV2_HIP_ERROR, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (!p) return fail(SDV2_HIP_ERROR, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SDV2_OK;
}
}  // namespace

extern "C" {

size_t sdv2_gemm_noalloc_max_scratch_bytes(void) { return kNoAllocScratchBytes; }

int32_t sdv2_gemm_bf16_noalloc(const void* a_dev, const void* w_dev, const float* bias_dev, void* out_dev, int32_t M,
                               int32_t N, int32_t K, int32_t epilogue, const float* gate_a_dev, const float* gate_b_dev,
                               int32_t gate_b_stride, int32_t rows_per_gate, void* hip_stream) {
    if (M <= 0 || N <= 0 || K <= 0 || epilogue < 0 || epilogue > 3) return fail(SDV2_INVALID_ARG, "bad M, N, K or epilogue");
    const size_t need = gemm_splitk_floats(M, N, K, epilogue) * sizeof(float);
    if (need > kNoAllocScratchBytes)
        return fail(SDV2_INVALID_ARG, "this shape's k-split needs %zu bytes of scratch, more than the built-in %zu: use "
                    "sdv2_gemm_bf16 with a workspace", need, (size_t)kNoAllocScratchBytes);
    void* ptr = nullptr;
    if (need) {
        const int32_t rc = noalloc_scratch(&ptr);
        if (rc) return rc;
    }
    return sdv2_gemm_bf16(a_dev, w_dev, bias_dev, out_dev, M, N, K, epilogue, gate_a_dev, gate_b_dev, gate_b_stride,
                          rows_per_gate, ptr, need ? kNoAllocScratchBytes : 0, hip_stream);
}

size_t sdv2_attention_workspace_bytes(int32_t B, int32_t L, int32_t C, int32_t max_kv_len) {
    if (B <= 0 || L <= 0 || C <= 0 || C % SDV2_HEAD_DIM || max_kv_len <= 0) return 0;
    return align_up(attention_workspace_bytes(B, L, C, max_kv_len), 256);
}

int32_t sdv2_attention_bf16(const void* q_dev, const void* const* k_dev, const void* const* vt_dev,
                            const int32_t* kv_len_host, const int32_t* cap_host, void* o_dev, int32_t B, int32_t L,
                            int32_t n_heads, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    if (!q_dev || !k_dev || !vt_dev || !kv_len_host || !cap_host || !o_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    if (B <= 0 || B > SDV2_MAX_BATCH || L <= 0 || n_heads <= 0) return fail(SDV2_INVALID_ARG, "bad B, L or n_heads");
    AttnArgs a;
    memset(&a, 0, sizeof(a));
    int max_kv = 0;
    for (int b = 0; b < B; ++b) {
        if (!k_dev[b] || !vt_dev[b]) return fail(SDV2_INVALID_ARG, "null K/V of stream %d", b);
        if (kv_len_host[b] <= 0 || cap_host[b] % 64 || cap_host[b] < kv_len_host[b])
            return fail(SDV2_INVALID_ARG, "stream %d: need 0 < kv_len <= cap, cap multiple of 64", b);
        a.k[b] = static_cast<const bf16*>(k_dev[b]);
        a.vt[b] = static_cast<const bf16*>(vt_dev[b]);
        a.kv_len[b] = kv_len_host[b];
        a.cap[b] = cap_host[b];
        if (kv_len_host[b] > max_kv) max_kv = kv_len_host[b];
    }
    const int C = n_heads * SDV2_HEAD_DIM;
    a.splits = attention_plan_splits(B, L, n_heads, max_kv);
    const size_t need = align_up(attention_workspace_bytes(B, L, C, max_kv), 256);
    if (need > 0 && (!workspace_dev || workspace_bytes < need))
        return fail(SDV2_WORKSPACE_TOO_SMALL, "attention workspace %zu < %zu", workspace_bytes, need);
    a.q = static_cast<const bf16*>(q_dev);
    a.o = static_cast<bf16*>(o_dev);
    a.B = B;
    a.L = L;
    a.H = n_heads;
    a.part_o = static_cast<float*>(workspace_dev);
    a.part_ml = a.part_o ? a.part_o + (size_t)a.splits * B * L * C : nullptr;
    HIP_TRY(launch_attention(a, static_cast<hipStream_t>(hip_stream)), "attention kernel");
    return SDV2_OK;
}

// ------------------------------------------------------------------------------------------ text K/V
size_t sdv2_text_kv_bytes(const sdv2_model_cfg* cfg) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) {
        fail(SDV2_INVALID_ARG, "%s", why);
        return 0;
    }
    return align_up((size_t)cfg->text_len, 64) * cfg->C * sizeof(bf16);
}

size_t sdv2_text_kv_workspace_bytes(const sdv2_model_cfg* cfg) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) {
        fail(SDV2_INVALID_ARG, "%s", why);
        return 0;
    }
    return 2 * align_up((size_t)cfg->text_len * cfg->C * sizeof(bf16), 256);
}

int32_t sdv2_text_kv_prepare(const sdv2_model_cfg* cfg, const sdv2_block_weights* w, const void* ctx_dev,
                             void* kt_dev, void* vtt_dev, void* workspace_dev, size_t workspace_bytes,
                             void* hip_stream) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!w || w->struct_size != sizeof(sdv2_block_weights)) return fail(SDV2_INVALID_ARG, "bad block weights");
    if (!w->W_ck || !w->b_ck || !w->g_ck || !w->W_cv || !w->b_cv) return fail(SDV2_INVALID_ARG, "text K/V weights missing");
    if (!ctx_dev || !kt_dev || !vtt_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    const size_t need = sdv2_text_kv_workspace_bytes(cfg);
    if (workspace_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, need);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int C = cfg->C, Lt = cfg->text_len;
    bf16* krows = static_cast<bf16*>(workspace_dev);
    bf16* vrows = reinterpret_cast<bf16*>(static_cast<unsigned char*>(workspace_dev) + need / 2);
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.a = static_cast<const bf16*>(ctx_dev);
    g.M = Lt;
    g.N = C;
    g.K = C;
    g.epilogue = kEpiBias;
    g.rows_per_gate = 1;
    g.w = static_cast<const bf16*>(w->W_ck);
    g.bias = w->b_ck;
    g.out = krows;
    HIP_TRY(launch_gemm(g, s), "text K gemm");
    HIP_TRY(launch_rmsnorm_inplace(krows, w->g_ck, Lt, C, C, cfg->eps, s), "text K norm");
    g.w = static_cast<const bf16*>(w->W_cv);
    g.bias = w->b_cv;
    g.out = vrows;
    HIP_TRY(launch_gemm(g, s), "text V gemm");
    HIP_TRY(launch_text_relayout(krows, vrows, static_cast<bf16*>(kt_dev), static_cast<bf16*>(vtt_dev), Lt, C,
                                 cfg->n_heads, (int)align_up((size_t)Lt, 64), s),
            "text relayout");
    return SDV2_OK;
}

// ------------------------------------------------------------------------------------------ conditioning
size_t sdv2_conditioning_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B) {
    const char* why;
    if (!model_cfg_ok(cfg, &why) || B <= 0 || B > SDV2_MAX_BATCH) {
        fail(SDV2_INVALID_ARG, "bad cfg or B");
        return 0;
    }
    return align_up((size_t)B * cfg->t_dim * 4, 256) + 2 * align_up((size_t)B * cfg->C * 4, 256);
}

}  // extern "C"

namespace {
// desc (device) replaces timesteps_host when the launches are recorded into a graph
int32_t conditioning_impl(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, int32_t B,
                          const float* timesteps_host, const float* tvec_dev, const StepDesc* desc, float* e0_dev,
                          void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (B <= 0 || B > SDV2_MAX_BATCH) return fail(SDV2_INVALID_ARG, "B = %d out of range", B);
    if (!mw || mw->struct_size != sizeof(sdv2_model_weights)) return fail(SDV2_INVALID_ARG, "bad model weights");
    if (desc != nullptr) timesteps_host = reinterpret_cast<const float*>(desc);      // only its being non-null matters below
    if ((timesteps_host == nullptr) == (tvec_dev == nullptr))
        return fail(SDV2_INVALID_ARG, "give exactly one of timesteps_host and tvec_dev");
    if (!e0_dev || !mw->W_mod || !mw->b_mod) return fail(SDV2_INVALID_ARG, "null pointer");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int C = cfg->C;
    const float* tvec = tvec_dev;
    if (timesteps_host) {
        if (!mw->W_t1 || !mw->b_t1 || !mw->W_t2 || !mw->b_t2) return fail(SDV2_INVALID_ARG, "timestep MLP weights missing");
        const size_t need = sdv2_conditioning_workspace_bytes(cfg, B);
        if (!workspace_dev || workspace_bytes < need)
            return fail(SDV2_WORKSPACE_TOO_SMALL, "conditioning workspace %zu < %zu", workspace_bytes, need);
        unsigned char* p = static_cast<unsigned char*>(workspace_dev);
        float* emb = reinterpret_cast<float*>(p);
        p += align_up((size_t)B * cfg->t_dim * 4, 256);
        float* a1 = reinterpret_cast<float*>(p);
        p += align_up((size_t)B * C * 4, 256);
        float* tv = reinterpret_cast<float*>(p);
        HIP_TRY(launch_timestep_embedding(desc ? nullptr : timesteps_host, desc, emb, B, cfg->t_dim, (double)cfg->rope_base, s),
                "timestep embedding");
        HIP_TRY(launch_gemv(emb, static_cast<const bf16*>(mw->W_t1), mw->b_t1, a1, B, C, cfg->t_dim, 0, s), "timestep MLP 1");
        HIP_TRY(launch_gemv(a1, static_cast<const bf16*>(mw->W_t2), mw->b_t2, tv, B, C, C, 1, s), "timestep MLP 2");
        tvec = tv;
    }
    HIP_TRY(launch_gemv(tvec, static_cast<const bf16*>(mw->W_mod), mw->b_mod, e0_dev, B, 6 * C, C, 1, s), "modulation projection");
    return SDV2_OK;
}
}  // namespace

extern "C" {

int32_t sdv2_conditioning(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, int32_t B,
                          const float* timesteps_host, const float* tvec_dev, float* e0_dev, void* workspace_dev,
                          size_t workspace_bytes, void* hip_stream) {
    return conditioning_impl(cfg, mw, B, timesteps_host, tvec_dev, nullptr, e0_dev, workspace_dev, workspace_bytes, hip_stream);
}

}  // extern "C"

// ------------------------------------------------------------------------------------------ the block
namespace {

struct BlockWorkspace {
    bf16* h;        // [rows, C]
    bf16* qkv;      // [rows, 3C]
    bf16* q;        // [rows, C]
    bf16* o;        // [rows, C]
    bf16* u;        // [rows, F]
    float* attn;    // split-KV partials
    size_t attn_bytes;
    float* gemm_partials;   // split-K partial sums
    size_t gemm_floats;
    size_t total;
};

BlockWorkspace carve_block(const sdv2_model_cfg* cfg, int B, int L, int max_kv, unsigned char* base) {
    const size_t rows = (size_t)B * L;
    const size_t C = cfg->C, F = cfg->ffn_dim;
    BlockWorkspace w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        unsigned char* p = base ? base + off : nullptr;
        off += align_up(bytes, 256);
        return p;
    };
    w.h = reinterpret_cast<bf16*>(take(rows * C * 2));
    w.qkv = reinterpret_cast<bf16*>(take(rows * 3 * C * 2));
    w.q = reinterpret_cast<bf16*>(take(rows * C * 2));
    w.o = reinterpret_cast<bf16*>(take(rows * C * 2));
    w.u = reinterpret_cast<bf16*>(take(rows * F * 2));
    const size_t a1 = attention_workspace_bytes(B, L, (int)C, max_kv);
    const size_t a2 = attention_workspace_bytes(B, L, (int)C, cfg->text_len);
    w.attn_bytes = a1 > a2 ? a1 : a2;
    w.attn = reinterpret_cast<float*>(take(w.attn_bytes));
    // split-K room for the largest need among the block's six projections
    const int shapes[6][3] = {{(int)(3 * C), (int)C, kEpiBias}, {(int)C, (int)C, kEpiGatedResidual}, {(int)C, (int)C, kEpiBias},
                              {(int)C, (int)C, kEpiResidual},   {(int)F, (int)C, kEpiBiasGelu},      {(int)C, (int)F, kEpiGatedResidual}};
    w.gemm_floats = 0;
    for (const auto& sh : shapes) {
        const size_t f = gemm_splitk_floats((int)rows, sh[0], sh[1], sh[2]);
        if (f > w.gemm_floats) w.gemm_floats = f;
    }
    w.gemm_partials = reinterpret_cast<float*>(take(w.gemm_floats * sizeof(float)));
    w.total = off;
    return w;
}

// Everything that can be rejected without touching state.  Fills per-stream L and returns it.
int32_t validate_block_call(const sdv2_model_cfg* cfg, const sdv2_block_weights* w, const sdv2_kv_cache* cache,
                            int32_t layer, const sdv2_chunk_desc* chunks, int32_t B, int* L_out) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!w || w->struct_size != sizeof(sdv2_block_weights)) return fail(SDV2_INVALID_ARG, "bad block weights (layer %d)", layer);
    const void* need[] = {w->W_qkv, w->b_qkv, w->g_q, w->g_k, w->W_o, w->b_o, w->mod_table, w->ln3_gamma, w->ln3_beta,
                          w->W_cq, w->b_cq, w->g_cq, w->W_co, w->b_co, w->W_1, w->b_1, w->W_2, w->b_2};
    for (const void* p : need)
        if (!p) return fail(SDV2_INVALID_ARG, "a weight pointer of layer %d is null", layer);
    if (!cache) return fail(SDV2_INVALID_ARG, "cache handle is null");
    if (layer < 0 || layer >= cache->cfg.n_layers) return fail(SDV2_INVALID_ARG, "layer %d out of range", layer);
    if (cache->cfg.n_heads != cfg->n_heads || cache->cfg.tokens_per_frame != cfg->grid_h * cfg->grid_w)
        return fail(SDV2_INVALID_ARG, "cache and model shapes disagree");
    if (B < 1 || B > SDV2_MAX_BATCH) return fail(SDV2_INVALID_ARG, "B = %d out of range", B);
    if (!chunks) return fail(SDV2_INVALID_ARG, "chunks is null");
    const int P = cfg->grid_h * cfg->grid_w;
    for (int b = 0; b < B; ++b) {
        const sdv2_chunk_desc& c = chunks[b];
        if (c.stream_id < 0 || c.stream_id >= cache->cfg.n_streams) return fail(SDV2_INVALID_ARG, "stream %d out of range", c.stream_id);
        for (int j = 0; j < b; ++j)
            if (chunks[j].stream_id == c.stream_id) return fail(SDV2_INVALID_ARG, "stream %d listed twice", c.stream_id);
        if (c.n_frames <= 0 || c.n_frames != chunks[0].n_frames) return fail(SDV2_INVALID_ARG, "n_frames must be positive and equal across streams");
        if ((int64_t)c.n_frames * P > cache->cfg.window_tokens) return fail(SDV2_INVALID_ARG, "chunk larger than the window");
        if (c.frame_pos0 < 0) return fail(SDV2_INVALID_ARG, "frame_pos0 < 0");
        const size_t idx = (size_t)layer * cache->cfg.n_streams + c.stream_id;
        if (!c.advance && cache->last_n[idx] != c.n_frames * P)
            return fail(SDV2_BAD_STATE, "stream %d layer %d: advance = 0 without a matching append", c.stream_id, layer);
    }
    *L_out = chunks[0].n_frames * P;
    return SDV2_OK;
}

void fill_rope_table(const sdv2_model_cfg* cfg, RopeAppendArgs* a) {
    const int pairs = SDV2_HEAD_DIM / 2;
    const int third = pairs / 3;
    const int counts[3] = {pairs - 2 * third, third, third};
    int p = 0;
    for (int axis = 0; axis < 3; ++axis)
        for (int j = 0; j < counts[axis]; ++j, ++p) {
            a->pair_axis[p] = axis;
            a->inv_freq[p] = pow((double)cfg->rope_base, -(double)j / counts[axis]);
        }
}

// Launches one block.  State has been validated; it is advanced here and restored if a launch fails.
// next_w: the block that runs next on the same x and workspace (null: none); when FFN-2's k-split reduce pass could
// also write that block's adaLN-1 output into ws.h, *next_h_ready is set and the next call passes h_ready = true.
// desc: null for an ordinary call.  Otherwise the launches are being recorded into a graph: the host ring state is
// left alone, the kernels read token ids, frame positions and key counts from *desc (device memory) at run time, and
// the attention plan is the one of a full cache.
int32_t run_block(const sdv2_model_cfg* cfg, const sdv2_block_weights* w, sdv2_kv_cache* cache, int layer, float* x,
                  const float* e0, const void* const* kt, const void* const* vtt, const sdv2_chunk_desc* chunks, int B,
                  int L, const BlockWorkspace& ws, hipStream_t s, const sdv2_block_weights* next_w = nullptr,
                  bool h_ready = false, bool* next_h_ready = nullptr, const StepDesc* desc = nullptr) {
    const int C = cfg->C, F = cfg->ffn_dim, H = cfg->n_heads;
    const int rows = B * L;
    const int S = cache->cfg.sink_tokens, W = cache->cfg.window_tokens;
    int64_t old_total[SDV2_MAX_BATCH];
    int32_t old_last[SDV2_MAX_BATCH];
    RopeAppendArgs ra;
    memset(&ra, 0, sizeof(ra));
    AttnArgs at;
    memset(&at, 0, sizeof(at));
    int max_kv = 0;
    for (int b = 0; b < B; ++b) {
        const size_t idx = (size_t)layer * cache->cfg.n_streams + chunks[b].stream_id;
        old_total[b] = cache->total[idx];
        old_last[b] = cache->last_n[idx];
        if (desc == nullptr && chunks[b].advance) {
            cache->total[idx] += L;
            cache->last_n[idx] = L;
        }
        ra.st[b] = append_stream(cache, layer, chunks[b].stream_id, desc ? 0 : cache->total[idx] - L, chunks[b].frame_pos0);
        at.k[b] = ra.st[b].k_cache;
        at.vt[b] = ra.st[b].vt_cache;
        const int64_t res = (desc == nullptr && cache->total[idx] < (int64_t)S + W) ? cache->total[idx] : (int64_t)S + W;
        at.kv_len[b] = (int)res;
        at.cap[b] = cache->cap;
        if (at.kv_len[b] > max_kv) max_kv = at.kv_len[b];
    }
    ra.desc = desc;
    at.desc = desc;
    auto restore = [&]() {
        if (desc != nullptr) return;
        for (int b = 0; b < B; ++b) {
            const size_t idx = (size_t)layer * cache->cfg.n_streams + chunks[b].stream_id;
            cache->total[idx] = old_total[b];
            cache->last_n[idx] = old_last[b];
        }
    };
#define RUN(tag, expr, what)                                              \
    do {                                                                  \
        hipError_t e__ = timed(tag, s, [&]() { return (expr); });         \
        if (e__ != hipSuccess) {                                          \
            restore();                                                    \
            return hip_fail(e__, what);                                   \
        }                                                                 \
    } while (0)

    // a product on the matrix cores and its second pass (the sum of the k parts; the merge of a split key range) are
    // timed as two launches
#define RUN_GEMM(tag, what)                                                         \
    do {                                                                            \
        RUN(tag, launch_gemm_part(g, s, 1), what);                                  \
        if (gemm_splits_k(g)) RUN(SDV2_TAG_GEMM_REDUCE, launch_gemm_part(g, s, 2), what " (sum of the k parts)"); \
    } while (0)
#define RUN_ATTN(tag, args, what)                                                   \
    do {                                                                            \
        RUN(tag, launch_attention(args, s, 1), what);                               \
        if (attention_has_merge_pass(args)) RUN(SDV2_TAG_ATTN_MERGE, launch_attention(args, s, 2), what " (merge)"); \
    } while (0)

    const float* tab = w->mod_table;
    LnArgs ln;
    ln.x = x;
    ln.out = ws.h;
    ln.rows = rows;
    ln.C = C;
    ln.eps = cfg->eps;
    ln.b_stride = 6 * C;
    ln.rows_per_stream = L;
    // 1. adaLN-1
    ln.shift_a = tab + 0 * C;
    ln.shift_b = e0 + 0 * C;
    ln.scale_a = tab + 1 * C;
    ln.scale_b = e0 + 1 * C;
    if (!h_ready) RUN(SDV2_TAG_ADALN1, launch_layernorm(ln, s), "adaLN-1");
    // 2. QKV projection
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.splitk_partials = ws.gemm_floats ? ws.gemm_partials : nullptr;
    g.splitk_floats = ws.gemm_floats;
    g.M = rows;
    g.rows_per_gate = L;
    g.gate_b_stride = 6 * C;
    g.a = ws.h;
    g.w = static_cast<const bf16*>(w->W_qkv);
    g.bias = w->b_qkv;
    g.out = ws.qkv;
    g.N = 3 * C;
    g.K = C;
    g.epilogue = kEpiBias;
    RUN_GEMM(SDV2_TAG_QKV, "QKV gemm");
    // 3. q/k RMSNorm + RoPE + append into the ring
    ra.qkv = ws.qkv;
    ra.q_out = ws.q;
    ra.g_q = w->g_q;
    ra.g_k = w->g_k;
    ra.B = B;
    ra.L = L;
    ra.C = C;
    ra.H = H;
    ra.tokens_per_frame = cfg->grid_h * cfg->grid_w;
    ra.grid_w = cfg->grid_w;
    ra.S = S;
    ra.W = W;
    ra.eps = cfg->eps;
    fill_rope_table(cfg, &ra);
    RUN(SDV2_TAG_ROPE_APPEND, launch_rope_append(ra, s), "rope + append");
    // 4. self-attention over every resident slot
    at.q = ws.q;
    at.o = ws.o;
    at.B = B;
    at.L = L;
    at.H = H;
    at.splits = attention_plan_splits(B, L, H, max_kv);
    at.part_o = ws.attn;
    at.part_ml = ws.attn + (size_t)at.splits * rows * C;
    RUN_ATTN(SDV2_TAG_SELF_ATTN, at, "self-attention");
    // 5. output projection, gated residual
    g.a = ws.o;
    g.w = static_cast<const bf16*>(w->W_o);
    g.bias = w->b_o;
    g.out = x;
    g.N = C;
    g.K = C;
    g.epilogue = kEpiGatedResidual;
    g.gate_a = tab + 2 * C;
    g.gate_b = e0 + 2 * C;
    RUN_GEMM(SDV2_TAG_OUT_PROJ, "out-proj gemm");
    // 6. LayerNorm-3 (affine) and the cross-attention query
    ln.scale_a = w->ln3_gamma;
    ln.scale_b = nullptr;
    ln.shift_a = w->ln3_beta;
    ln.shift_b = nullptr;
    RUN(SDV2_TAG_LN3, launch_layernorm(ln, s), "LN-3");
    g.a = ws.h;
    g.w = static_cast<const bf16*>(w->W_cq);
    g.bias = w->b_cq;
    g.out = ws.q;
    g.epilogue = kEpiBias;
    RUN_GEMM(SDV2_TAG_CROSS_Q, "cross-q gemm");
    RUN(SDV2_TAG_CROSS_Q_NORM, launch_rmsnorm_inplace(ws.q, w->g_cq, rows, C, C, cfg->eps, s), "cross-q norm");
    // 7. cross-attention over the text tokens
    AttnArgs ct = at;
    ct.desc = nullptr;                                // the text keys do not change from step to step
    const int cap_t = (int)align_up((size_t)cfg->text_len, 64);
    for (int b = 0; b < B; ++b) {
        ct.k[b] = static_cast<const bf16*>(kt[b]);
        ct.vt[b] = static_cast<const bf16*>(vtt[b]);
        ct.kv_len[b] = cfg->text_len;
        ct.cap[b] = cap_t;
    }
    ct.splits = attention_plan_splits(B, L, H, cfg->text_len);
    ct.part_ml = ws.attn + (size_t)ct.splits * rows * C;
    RUN_ATTN(SDV2_TAG_CROSS_ATTN, ct, "cross-attention");
    g.a = ws.o;
    g.w = static_cast<const bf16*>(w->W_co);
    g.bias = w->b_co;
    g.out = x;
    g.epilogue = kEpiResidual;
    RUN_GEMM(SDV2_TAG_CROSS_OUT, "cross-out gemm");
    // 8. adaLN-2 and the FFN
    ln.shift_a = tab + 3 * C;
    ln.shift_b = e0 + 3 * C;
    ln.scale_a = tab + 4 * C;
    ln.scale_b = e0 + 4 * C;
    RUN(SDV2_TAG_ADALN2, launch_layernorm(ln, s), "adaLN-2");
    g.a = ws.h;
    g.w = static_cast<const bf16*>(w->W_1);
    g.bias = w->b_1;
    g.out = ws.u;
    g.N = F;
    g.K = C;
    g.epilogue = kEpiBiasGelu;
    RUN_GEMM(SDV2_TAG_FFN1, "FFN-1 gemm");
    g.a = ws.u;
    g.w = static_cast<const bf16*>(w->W_2);
    g.bias = w->b_2;
    g.out = x;
    g.N = C;
    g.K = F;
    g.epilogue = kEpiGatedResidual;
    g.gate_a = tab + 5 * C;
    g.gate_b = e0 + 5 * C;
    if (next_w != nullptr && next_h_ready != nullptr) {
        LnArgs ln1 = ln;                             // the next block's adaLN-1 on the x this product completes
        ln1.shift_a = next_w->mod_table + 0 * C;
        ln1.shift_b = e0 + 0 * C;
        ln1.scale_a = next_w->mod_table + 1 * C;
        ln1.scale_b = e0 + 1 * C;
        RUN(SDV2_TAG_FFN2, launch_gemm_then_layernorm(g, ln1, next_h_ready, s, 1), "FFN-2 gemm");
        if (gemm_splits_k(g))
            RUN(SDV2_TAG_GEMM_REDUCE, launch_gemm_then_layernorm(g, ln1, next_h_ready, s, 2), "FFN-2 gemm (sum of the k parts)");
    } else {
        RUN_GEMM(SDV2_TAG_FFN2, "FFN-2 gemm");
    }
#undef RUN_GEMM
#undef RUN_ATTN
#undef RUN
    return SDV2_OK;
}

int max_kv_possible(const sdv2_kv_cache* cache) { return cache->cfg.sink_tokens + cache->cfg.window_tokens; }

}  // namespace

extern "C" {

size_t sdv2_block_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L) {
    const char* why;
    if (!model_cfg_ok(cfg, &why) || B <= 0 || B > SDV2_MAX_BATCH || L <= 0) {
        fail(SDV2_INVALID_ARG, "bad cfg, B or L");
        return 0;
    }
    // sized for the largest split plan any cache length can ask for
    size_t worst = 0;
    for (int kv = 64; kv <= (1 << 20); kv *= 2) {
        const size_t t = carve_block(cfg, B, L, kv, nullptr).total;
        if (t > worst) worst = t;
    }
    return worst;
}

int32_t sdv2_dit_block_forward(const sdv2_model_cfg* cfg, const sdv2_block_weights* w, sdv2_kv_cache* cache,
                               int32_t layer, float* x_dev, const float* e0_dev, const void* const* kt_dev,
                               const void* const* vtt_dev, const sdv2_chunk_desc* chunks, int32_t B,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    int L = 0;
    int32_t rc = validate_block_call(cfg, w, cache, layer, chunks, B, &L);
    if (rc) return rc;
    if (!x_dev || !e0_dev || !kt_dev || !vtt_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    for (int b = 0; b < B; ++b)
        if (!kt_dev[b] || !vtt_dev[b]) return fail(SDV2_INVALID_ARG, "text K/V of stream slot %d is null", b);
    const size_t need = sdv2_block_workspace_bytes(cfg, B, L);
    if (workspace_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, need);
    const BlockWorkspace ws = carve_block(cfg, B, L, max_kv_possible(cache), static_cast<unsigned char*>(workspace_dev));
    return run_block(cfg, w, cache, layer, x_dev, e0_dev, kt_dev, vtt_dev, chunks, B, L, ws,
                     static_cast<hipStream_t>(hip_stream));
}

size_t sdv2_denoise_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L) {
    const size_t blk = sdv2_block_workspace_bytes(cfg, B, L);
    if (!blk) return 0;
    return blk + align_up((size_t)B * 6 * cfg->C * 4, 256) + sdv2_conditioning_workspace_bytes(cfg, B);
}

}  // extern "C"

namespace {
// sdv2_denoise_step; with desc non-null the launches are being recorded into a graph (see run_block)
int32_t denoise_impl(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, sdv2_kv_cache* cache, float* x_dev,
                     const float* timesteps_host, const float* tvec_dev, const void* const* kt_dev,
                     const void* const* vtt_dev, const sdv2_chunk_desc* chunks, int32_t B, void* workspace_dev,
                     size_t workspace_bytes, void* hip_stream, const StepDesc* desc) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!mw || mw->struct_size != sizeof(sdv2_model_weights) || !mw->blocks) return fail(SDV2_INVALID_ARG, "bad model weights");
    if (!cache || cache->cfg.n_layers != cfg->n_layers) return fail(SDV2_INVALID_ARG, "cache and model layer counts disagree");
    if (desc == nullptr && (timesteps_host == nullptr) == (tvec_dev == nullptr))
        return fail(SDV2_INVALID_ARG, "give exactly one of timesteps_host and tvec_dev");
    if (!x_dev || !kt_dev || !vtt_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    int L = 0;
    for (int layer = 0; layer < cfg->n_layers; ++layer) {
        int32_t rc = validate_block_call(cfg, &mw->blocks[layer], cache, layer, chunks, B, &L);
        if (rc) return rc;
        for (int b = 0; b < B; ++b)
            if (!kt_dev[(size_t)layer * B + b] || !vtt_dev[(size_t)layer * B + b])
                return fail(SDV2_INVALID_ARG, "text K/V of layer %d slot %d is null", layer, b);
    }
    const size_t need = sdv2_denoise_workspace_bytes(cfg, B, L);
    if (workspace_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, need);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned char* p = static_cast<unsigned char*>(workspace_dev);
    const size_t blk = sdv2_block_workspace_bytes(cfg, B, L);
    float* e0 = reinterpret_cast<float*>(p + blk);
    void* cond_ws = p + blk + align_up((size_t)B * 6 * cfg->C * 4, 256);
    int32_t rc = conditioning_impl(cfg, mw, B, timesteps_host, tvec_dev, desc, e0, cond_ws,
                                   sdv2_conditioning_workspace_bytes(cfg, B), hip_stream);
    if (rc) return rc;
    const BlockWorkspace ws = carve_block(cfg, B, L, max_kv_possible(cache), p);
    // Ring positions of every layer of the listed streams, to put back if a launch fails half way: the layers that
    // already ran would otherwise sit one chunk ahead of the others.  (x and the cache contents of those layers have
    // been overwritten by then; the call reports the failing layer.)
    std::vector<int64_t> total0((size_t)cfg->n_layers * B);
    std::vector<int32_t> last0((size_t)cfg->n_layers * B);
    for (int layer = 0; layer < cfg->n_layers; ++layer)
        for (int b = 0; b < B; ++b) {
            const size_t idx = (size_t)layer * cache->cfg.n_streams + chunks[b].stream_id;
            total0[(size_t)layer * B + b] = cache->total[idx];
            last0[(size_t)layer * B + b] = cache->last_n[idx];
        }
    bool h_ready = false;
    for (int layer = 0; layer < cfg->n_layers; ++layer) {
        bool next_ready = false;
        rc = run_block(cfg, &mw->blocks[layer], cache, layer, x_dev, e0, kt_dev + (size_t)layer * B,
                       vtt_dev + (size_t)layer * B, chunks, B, L, ws, s,
                       layer + 1 < cfg->n_layers ? &mw->blocks[layer + 1] : nullptr, h_ready, &next_ready, desc);
        h_ready = next_ready;
        if (rc) {
            for (int l2 = 0; l2 < layer; ++l2)
                for (int b = 0; b < B; ++b) {
                    const size_t idx = (size_t)l2 * cache->cfg.n_streams + chunks[b].stream_id;
                    cache->total[idx] = total0[(size_t)l2 * B + b];
                    cache->last_n[idx] = last0[(size_t)l2 * B + b];
                }
            const std::string inner = g_last_error;
            return fail(rc, "layer %d: %s", layer, inner.c_str());
        }
    }
    return SDV2_OK;
}
}  // namespace

// ------------------------------------------------------------------------------------------ the step as a replayed graph
struct sdv2_denoise_graph {
    sdv2_model_cfg cfg;
    sdv2_kv_cache* cache;
    int B, n_frames, L;
    int32_t stream_ids[SDV2_MAX_BATCH];
    StepDesc* desc_dev;
    hipStream_t capture_stream;
    hipGraph_t graph;
    hipGraphExec_t exec;
};

extern "C" {

int32_t sdv2_denoise_step(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, sdv2_kv_cache* cache, float* x_dev,
                          const float* timesteps_host, const float* tvec_dev, const void* const* kt_dev,
                          const void* const* vtt_dev, const sdv2_chunk_desc* chunks, int32_t B, void* workspace_dev,
                          size_t workspace_bytes, void* hip_stream) {
    return denoise_impl(cfg, mw, cache, x_dev, timesteps_host, tvec_dev, kt_dev, vtt_dev, chunks, B, workspace_dev,
                        workspace_bytes, hip_stream, nullptr);
}

size_t sdv2_denoise_graph_state_bytes(void) { return align_up(sizeof(StepDesc), 256); }

int32_t sdv2_denoise_graph_create(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, sdv2_kv_cache* cache,
                                  float* x_dev, const void* const* kt_dev, const void* const* vtt_dev,
                                  const int32_t* stream_ids, int32_t B, int32_t n_frames, void* workspace_dev,
                                  size_t workspace_bytes, void* state_dev, size_t state_bytes, sdv2_denoise_graph** out) {
    if (!out || !stream_ids || !state_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    if (state_bytes < sdv2_denoise_graph_state_bytes() || reinterpret_cast<uintptr_t>(state_dev) % 256)
        return fail(SDV2_INVALID_ARG, "state_dev must be 256-byte aligned and hold sdv2_denoise_graph_state_bytes() bytes");
    if (B < 1 || B > SDV2_MAX_BATCH || n_frames < 1) return fail(SDV2_INVALID_ARG, "bad B or n_frames");
    if (g_prof.on) return fail(SDV2_BAD_STATE, "per-launch profiling is on: its events cannot be recorded into a graph");
    sdv2_chunk_desc chunks[SDV2_MAX_BATCH];
    for (int b = 0; b < B; ++b) chunks[b] = sdv2_chunk_desc{stream_ids[b], 0, n_frames, 1};
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!mw || !mw->blocks || !cache) return fail(SDV2_INVALID_ARG, "null pointer");
    // every dense kernel of the step gets its attributes set before the capture begins
    {
        int L0 = 0;
        int32_t rc = validate_block_call(cfg, &mw->blocks[0], cache, 0, chunks, B, &L0);
        if (rc) return rc;
        const int C = cfg->C, F = cfg->ffn_dim, rows = B * L0;
        const BlockWorkspace ws = carve_block(cfg, B, L0, max_kv_possible(cache), nullptr);
        set_attributes_only(true);
        hipError_t e = hipSuccess;
        const int shapes[6][3] = {{3 * C, C, kEpiBias}, {C, C, kEpiGatedResidual}, {C, C, kEpiBias},
                                  {C, C, kEpiResidual}, {F, C, kEpiBiasGelu},      {C, F, kEpiGatedResidual}};
        for (const auto& sh : shapes) {
            GemmArgs g;
            memset(&g, 0, sizeof(g));
            g.M = rows;
            g.N = sh[0];
            g.K = sh[1];
            g.epilogue = sh[2];
            g.rows_per_gate = L0;
            g.splitk_partials = ws.gemm_floats ? reinterpret_cast<float*>(workspace_dev) : nullptr;   // only its being non-null matters
            g.splitk_floats = ws.gemm_floats;
            if (e == hipSuccess) e = launch_gemm(g, nullptr);
        }
        AttnArgs at;
        memset(&at, 0, sizeof(at));
        at.B = B;
        at.L = L0;
        at.H = cfg->n_heads;
        for (int b = 0; b < B; ++b) {
            at.kv_len[b] = max_kv_possible(cache);
            at.cap[b] = cache->cap;
        }
        at.splits = 1;
        if (e == hipSuccess) e = launch_attention(at, nullptr);
        set_attributes_only(false);
        if (e != hipSuccess) return hip_fail(e, "kernel attributes");
    }
    sdv2_denoise_graph* g = new (std::nothrow) sdv2_denoise_graph;
    if (!g) return fail(SDV2_INVALID_ARG, "out of host memory");
    g->cfg = *cfg;
    g->cache = cache;
    g->B = B;
    g->n_frames = n_frames;
    g->L = n_frames * cfg->grid_h * cfg->grid_w;
    for (int b = 0; b < SDV2_MAX_BATCH; ++b) g->stream_ids[b] = b < B ? stream_ids[b] : -1;
    g->desc_dev = static_cast<StepDesc*>(state_dev);
    g->graph = nullptr;
    g->exec = nullptr;
    hipError_t e = hipStreamCreateWithFlags(&g->capture_stream, hipStreamNonBlocking);
    if (e != hipSuccess) {
        delete g;
        return hip_fail(e, "hipStreamCreateWithFlags");
    }
    e = hipStreamBeginCapture(g->capture_stream, hipStreamCaptureModeRelaxed);
    if (e != hipSuccess) {
        hipStreamDestroy(g->capture_stream);
        delete g;
        return hip_fail(e, "hipStreamBeginCapture");
    }
    const int32_t rc = denoise_impl(cfg, mw, cache, x_dev, nullptr, nullptr, kt_dev, vtt_dev, chunks, B, workspace_dev,
                                    workspace_bytes, g->capture_stream, g->desc_dev);
    const std::string inner = g_last_error;
    e = hipStreamEndCapture(g->capture_stream, &g->graph);
    if (rc == SDV2_OK && e == hipSuccess) e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
    if (rc != SDV2_OK || e != hipSuccess) {
        if (g->graph) hipGraphDestroy(g->graph);
        hipStreamDestroy(g->capture_stream);
        delete g;
        if (rc != SDV2_OK) return fail(rc, "while recording the step: %s", inner.c_str());
        return hip_fail(e, "graph capture / instantiation");
    }
    *out = g;
    return SDV2_OK;
}

int32_t sdv2_denoise_graph_destroy(sdv2_denoise_graph* g) {
    if (!g) return SDV2_OK;
    if (g->exec) hipGraphExecDestroy(g->exec);
    if (g->graph) hipGraphDestroy(g->graph);
    hipStreamDestroy(g->capture_stream);
    delete g;
    return SDV2_OK;
}

int32_t sdv2_denoise_graph_launch(sdv2_denoise_graph* g, const float* timesteps_host, const sdv2_chunk_desc* chunks,
                                  int32_t B, void* hip_stream) {
    if (!g || !timesteps_host || !chunks) return fail(SDV2_INVALID_ARG, "null pointer");
    if (B != g->B) return fail(SDV2_INVALID_ARG, "B = %d, the graph was recorded for %d", B, g->B);
    sdv2_kv_cache* cache = g->cache;
    const sdv2_cache_cfg& cf = cache->cfg;
    const int L = g->L;
    const int64_t capacity = (int64_t)cf.sink_tokens + cf.window_tokens;
    StepDesc d;
    memset(&d, 0, sizeof(d));
    for (int b = 0; b < B; ++b) {
        const sdv2_chunk_desc& c = chunks[b];
        if (c.stream_id != g->stream_ids[b]) return fail(SDV2_INVALID_ARG, "slot %d: stream %d, the graph was recorded for stream %d", b, c.stream_id, g->stream_ids[b]);
        if (c.n_frames != g->n_frames) return fail(SDV2_INVALID_ARG, "n_frames differs from the recorded one");
        if (c.frame_pos0 < 0) return fail(SDV2_INVALID_ARG, "frame_pos0 < 0");
        const size_t idx0 = (size_t)c.stream_id;
        for (int layer = 1; layer < cf.n_layers; ++layer) {
            const size_t idx = (size_t)layer * cf.n_streams + c.stream_id;
            if (cache->total[idx] != cache->total[idx0] || cache->last_n[idx] != cache->last_n[idx0])
                return fail(SDV2_BAD_STATE, "stream %d: layer %d is not in step with layer 0", c.stream_id, layer);
        }
        if (!c.advance && cache->last_n[idx0] != L)
            return fail(SDV2_BAD_STATE, "stream %d: advance = 0 without a matching append", c.stream_id);
        const int64_t total_new = cache->total[idx0] + (c.advance ? L : 0);
        d.g0[b] = total_new - L;
        d.frame_pos0[b] = c.frame_pos0;
        d.kv_len[b] = (int)(total_new < capacity ? total_new : capacity);
        d.timestep[b] = timesteps_host[b];
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    HIP_TRY(launch_set_step_desc(d, g->desc_dev, s), "step descriptor kernel");
    HIP_TRY(hipGraphLaunch(g->exec, s), "hipGraphLaunch");
    for (int b = 0; b < B; ++b) {
        if (!chunks[b].advance) continue;
        for (int layer = 0; layer < cf.n_layers; ++layer) {
            const size_t idx = (size_t)layer * cf.n_streams + chunks[b].stream_id;
            cache->total[idx] += L;
            cache->last_n[idx] = L;
        }
    }
    return SDV2_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------ latents in, latents out
namespace {
bool io_weights_ok(const sdv2_io_weights* io) {
    return io && io->struct_size == sizeof(sdv2_io_weights) && io->W_pe && io->b_pe && io->head_table && io->W_head && io->b_head;
}
constexpr int kPatchWidth = 4 * kLatentChannels;      // numbers per token: 16 channels x 2 x 2 latent positions
}  // namespace

extern "C" {

int32_t sdv2_timestep_vector(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, int32_t B, const float* timesteps_host,
                             float* tvec_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (B <= 0 || B > SDV2_MAX_BATCH) return fail(SDV2_INVALID_ARG, "B = %d out of range", B);
    if (!mw || mw->struct_size != sizeof(sdv2_model_weights) || !mw->W_t1 || !mw->b_t1 || !mw->W_t2 || !mw->b_t2)
        return fail(SDV2_INVALID_ARG, "timestep MLP weights missing");
    if (!timesteps_host || !tvec_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    if (workspace_bytes < sdv2_conditioning_workspace_bytes(cfg, B)) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace too small");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned char* p = static_cast<unsigned char*>(workspace_dev);
    float* emb = reinterpret_cast<float*>(p);
    float* a1 = reinterpret_cast<float*>(p + align_up((size_t)B * cfg->t_dim * 4, 256));
    HIP_TRY(launch_timestep_embedding(timesteps_host, nullptr, emb, B, cfg->t_dim, (double)cfg->rope_base, s), "timestep embedding");
    HIP_TRY(launch_gemv(emb, static_cast<const bf16*>(mw->W_t1), mw->b_t1, a1, B, cfg->C, cfg->t_dim, 0, s), "timestep MLP 1");
    HIP_TRY(launch_gemv(a1, static_cast<const bf16*>(mw->W_t2), mw->b_t2, tvec_dev, B, cfg->C, cfg->C, 1, s), "timestep MLP 2");
    return SDV2_OK;
}

size_t sdv2_latent_io_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L) {
    const char* why;
    if (!model_cfg_ok(cfg, &why) || B <= 0 || B > SDV2_MAX_BATCH || L <= 0) {
        fail(SDV2_INVALID_ARG, "bad cfg, B or L");
        return 0;
    }
    // the larger of: bf16 patches; bf16 normalised rows + fp32 head output
    const size_t rows = (size_t)B * L;
    return align_up(rows * cfg->C * 2, 256) + align_up(rows * kPatchWidth * 4, 256);
}

int32_t sdv2_patch_embed(const sdv2_model_cfg* cfg, const sdv2_io_weights* io, const float* z_dev, int32_t B, int32_t n_frames,
                         float* x_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!io_weights_ok(io)) return fail(SDV2_INVALID_ARG, "bad io weights");
    if (B <= 0 || B > SDV2_MAX_BATCH || n_frames <= 0) return fail(SDV2_INVALID_ARG, "bad B or n_frames");
    if (!z_dev || !x_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    const int L = n_frames * cfg->grid_h * cfg->grid_w;
    if (workspace_bytes < sdv2_latent_io_workspace_bytes(cfg, B, L)) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace too small");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    bf16* patches = static_cast<bf16*>(workspace_dev);
    HIP_TRY(launch_patchify(z_dev, patches, B, n_frames, cfg->grid_h, cfg->grid_w, s), "patch gather");
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.a = patches;
    g.w = static_cast<const bf16*>(io->W_pe);
    g.bias = io->b_pe;
    g.out = x_dev;
    g.M = B * L;
    g.N = cfg->C;
    g.K = kPatchWidth;
    g.epilogue = kEpiPartial;                        // plain fp32 store of acc + bias
    g.rows_per_gate = 1;
    HIP_TRY(launch_gemm(g, s), "patch-embedding gemm");
    return SDV2_OK;
}

int32_t sdv2_output_head(const sdv2_model_cfg* cfg, const sdv2_io_weights* io, const float* x_dev, const float* tvec_dev,
                         int32_t B, int32_t n_frames, float* v_dev, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!io_weights_ok(io)) return fail(SDV2_INVALID_ARG, "bad io weights");
    if (B <= 0 || B > SDV2_MAX_BATCH || n_frames <= 0) return fail(SDV2_INVALID_ARG, "bad B or n_frames");
    if (!x_dev || !tvec_dev || !v_dev || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    const int L = n_frames * cfg->grid_h * cfg->grid_w, C = cfg->C;
    if (workspace_bytes < sdv2_latent_io_workspace_bytes(cfg, B, L)) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace too small");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned char* p = static_cast<unsigned char*>(workspace_dev);
    bf16* h = reinterpret_cast<bf16*>(p);
    float* tok = reinterpret_cast<float*>(p + align_up((size_t)B * L * C * 2, 256));
    LnArgs ln;
    ln.x = x_dev;
    ln.out = h;
    ln.rows = B * L;
    ln.C = C;
    ln.eps = cfg->eps;
    ln.shift_a = io->head_table;
    ln.scale_a = io->head_table + C;
    ln.shift_b = tvec_dev;
    ln.scale_b = tvec_dev;
    ln.b_stride = C;
    ln.rows_per_stream = L;
    HIP_TRY(launch_layernorm(ln, s), "head LayerNorm");
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.a = h;
    g.w = static_cast<const bf16*>(io->W_head);
    g.bias = io->b_head;
    g.out = tok;
    g.M = B * L;
    g.N = kPatchWidth;
    g.K = C;
    g.epilogue = kEpiPartial;
    g.rows_per_gate = 1;
    HIP_TRY(launch_gemm(g, s), "head gemm");
    HIP_TRY(launch_unpatchify(tok, v_dev, B, n_frames, cfg->grid_h, cfg->grid_w, s), "un-patching");
    return SDV2_OK;
}

int32_t sdv2_noise_latents(const float* x_dev, const float* eps_dev, float* out_dev, int32_t B, int64_t elems_per_stream,
                           const float* rate_host, void* hip_stream) {
    if (!x_dev || !eps_dev || !out_dev || !rate_host) return fail(SDV2_INVALID_ARG, "null pointer");
    if (B <= 0 || B > SDV2_MAX_BATCH || elems_per_stream <= 0) return fail(SDV2_INVALID_ARG, "bad B or size");
    for (int b = 0; b < B; ++b)
        if (!(rate_host[b] >= 0.0f && rate_host[b] <= 1.0f)) return fail(SDV2_INVALID_ARG, "noise rate of stream %d outside [0, 1]", b);
    HIP_TRY(launch_noise(x_dev, eps_dev, out_dev, B, elems_per_stream, rate_host, static_cast<hipStream_t>(hip_stream)), "noise kernel");
    return SDV2_OK;
}

int32_t sdv2_sampler_update(const float* z_dev, const float* v_dev, const float* eps_next_dev, float* z_next_dev, float* x0_dev,
                            int32_t B, int64_t elems_per_stream, const float* sigma_host, const float* sigma_next_host,
                            void* hip_stream) {
    if (!z_dev || !v_dev || !z_next_dev || !sigma_host || !sigma_next_host) return fail(SDV2_INVALID_ARG, "null pointer");
    if (B <= 0 || B > SDV2_MAX_BATCH || elems_per_stream <= 0) return fail(SDV2_INVALID_ARG, "bad B or size");
    for (int b = 0; b < B; ++b) {
        if (!(sigma_host[b] >= 0.0f && sigma_host[b] <= 1.0f) || !(sigma_next_host[b] >= 0.0f && sigma_next_host[b] <= sigma_host[b]))
            return fail(SDV2_INVALID_ARG, "stream %d: need 0 <= sigma_next <= sigma <= 1", b);
        if (sigma_next_host[b] > 0.0f && !eps_next_dev) return fail(SDV2_INVALID_ARG, "stream %d has a further step but eps_next is null", b);
    }
    HIP_TRY(launch_sampler(z_dev, v_dev, eps_next_dev, z_next_dev, x0_dev, B, elems_per_stream, sigma_host, sigma_next_host,
                           static_cast<hipStream_t>(hip_stream)), "sampler kernel");
    return SDV2_OK;
}

size_t sdv2_denoise_latents_workspace_bytes(const sdv2_model_cfg* cfg, int32_t B, int32_t L) {
    const size_t dn = sdv2_denoise_workspace_bytes(cfg, B, L);
    const size_t io = sdv2_latent_io_workspace_bytes(cfg, B, L);
    if (!dn || !io) return 0;
    const size_t rows = (size_t)B * L;
    return dn + io + align_up(rows * cfg->C * 4, 256) + align_up((size_t)B * cfg->C * 4, 256) + align_up(rows * kPatchWidth * 4, 256);
}

int32_t sdv2_denoise_latents_step(const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, const sdv2_io_weights* io,
                                  sdv2_kv_cache* cache, float* z_dev, const float* eps_next_dev, float* x0_dev,
                                  const float* sigma_host, const float* sigma_next_host, const void* const* kt_dev,
                                  const void* const* vtt_dev, const sdv2_chunk_desc* chunks, int32_t B, void* workspace_dev,
                                  size_t workspace_bytes, void* hip_stream) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!io_weights_ok(io)) return fail(SDV2_INVALID_ARG, "bad io weights");
    if (!z_dev || !sigma_host || !sigma_next_host || !chunks || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    if (B <= 0 || B > SDV2_MAX_BATCH) return fail(SDV2_INVALID_ARG, "B = %d out of range", B);
    float ts[SDV2_MAX_BATCH];
    for (int b = 0; b < B; ++b) {
        if (!(sigma_host[b] > 0.0f && sigma_host[b] <= 1.0f) || !(sigma_next_host[b] >= 0.0f && sigma_next_host[b] <= sigma_host[b]))
            return fail(SDV2_INVALID_ARG, "stream %d: need 0 <= sigma_next <= sigma, 0 < sigma <= 1", b);
        if (sigma_next_host[b] > 0.0f && !eps_next_dev) return fail(SDV2_INVALID_ARG, "stream %d has a further step but eps_next is null", b);
        if (chunks[b].n_frames != chunks[0].n_frames || chunks[b].n_frames <= 0) return fail(SDV2_INVALID_ARG, "n_frames must be positive and equal across streams");
        ts[b] = 1000.0f * sigma_host[b];
    }
    const int F = chunks[0].n_frames, L = F * cfg->grid_h * cfg->grid_w;
    const size_t need = sdv2_denoise_latents_workspace_bytes(cfg, B, L);
    if (!need || workspace_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, need);
    const size_t rows = (size_t)B * L;
    unsigned char* p = static_cast<unsigned char*>(workspace_dev);
    const size_t dn = sdv2_denoise_workspace_bytes(cfg, B, L), iob = sdv2_latent_io_workspace_bytes(cfg, B, L);
    void* dn_ws = p;
    void* io_ws = p + dn;
    float* x = reinterpret_cast<float*>(p + dn + iob);
    float* tvec = reinterpret_cast<float*>(p + dn + iob + align_up(rows * cfg->C * 4, 256));
    float* v = reinterpret_cast<float*>(p + dn + iob + align_up(rows * cfg->C * 4, 256) + align_up((size_t)B * cfg->C * 4, 256));
    // the cache-touching call comes first among the ones that can still refuse, so that a refusal leaves everything as it was
    int32_t rc = sdv2_timestep_vector(cfg, mw, B, ts, tvec, dn_ws, dn, hip_stream);
    if (rc) return rc;
    rc = sdv2_patch_embed(cfg, io, z_dev, B, F, x, io_ws, iob, hip_stream);
    if (rc) return rc;
    rc = sdv2_denoise_step(cfg, mw, cache, x, nullptr, tvec, kt_dev, vtt_dev, chunks, B, dn_ws, dn, hip_stream);
    if (rc) return rc;
    rc = sdv2_output_head(cfg, io, x, tvec, B, F, v, io_ws, iob, hip_stream);
    if (rc) return rc;
    return sdv2_sampler_update(z_dev, v, eps_next_dev, z_dev, x0_dev, B, (int64_t)kLatentChannels * F * 4 * cfg->grid_h * cfg->grid_w,
                               sigma_host, sigma_next_host, hip_stream);
}

}  // extern "C"

// ------------------------------------------------------------------------------------------ stream batch over denoising steps
struct sdv2_stream_batch {
    int n_steps, n_frames;
    size_t row_floats;                 // L * C
    float* x_pipe;                     // [n_steps][L][C], caller-owned
    int32_t cache_ids[SDV2_MAX_BATCH]; // cache stream of each depth
    int depth[SDV2_MAX_BATCH];         // per pipeline row: depth of the chunk it holds, -1 = free
    int32_t frame_pos0[SDV2_MAX_BATCH];
    int64_t entered;                   // chunks that have entered
    bool broken;
    int mode;                          // 0: not used yet; 1: rows are hidden states; 2: rows are latents
};

extern "C" {

size_t sdv2_stream_batch_rows_bytes(const sdv2_model_cfg* cfg, int32_t n_steps, int32_t n_frames) {
    const char* why;
    if (!model_cfg_ok(cfg, &why) || n_steps < 1 || n_steps > SDV2_MAX_BATCH || n_frames < 1) {
        fail(SDV2_INVALID_ARG, "bad cfg, n_steps or n_frames");
        return 0;
    }
    return align_up((size_t)n_steps * n_frames * cfg->grid_h * cfg->grid_w * cfg->C * sizeof(float), 256);
}

int32_t sdv2_stream_batch_create(const sdv2_model_cfg* cfg, int32_t n_steps, const int32_t* cache_stream_ids,
                                 int32_t n_frames, float* rows_dev, size_t rows_bytes, sdv2_stream_batch** out) {
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (n_steps < 1 || n_steps > SDV2_MAX_BATCH) return fail(SDV2_INVALID_ARG, "n_steps = %d outside 1 .. %d", n_steps, SDV2_MAX_BATCH);
    if (n_frames < 1) return fail(SDV2_INVALID_ARG, "n_frames must be positive");
    if (!cache_stream_ids || !rows_dev || !out) return fail(SDV2_INVALID_ARG, "null pointer");
    if (reinterpret_cast<uintptr_t>(rows_dev) % 256) return fail(SDV2_INVALID_ARG, "rows_dev must be 256-byte aligned");
    for (int d = 0; d < n_steps; ++d) {
        if (cache_stream_ids[d] < 0) return fail(SDV2_INVALID_ARG, "cache stream id of depth %d is negative", d);
        for (int e = 0; e < d; ++e)
            if (cache_stream_ids[e] == cache_stream_ids[d])
                return fail(SDV2_INVALID_ARG, "depths %d and %d name the same cache stream", e, d);
    }
    const size_t need = sdv2_stream_batch_rows_bytes(cfg, n_steps, n_frames);
    if (rows_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "rows buffer %zu < %zu", rows_bytes, need);
    sdv2_stream_batch* sb = new (std::nothrow) sdv2_stream_batch;
    if (!sb) return fail(SDV2_INVALID_ARG, "out of host memory");
    sb->n_steps = n_steps;
    sb->n_frames = n_frames;
    sb->row_floats = (size_t)n_frames * cfg->grid_h * cfg->grid_w * cfg->C;
    sb->x_pipe = rows_dev;
    for (int d = 0; d < SDV2_MAX_BATCH; ++d) {
        sb->cache_ids[d] = d < n_steps ? cache_stream_ids[d] : -1;
        sb->depth[d] = -1;
        sb->frame_pos0[d] = 0;
    }
    sb->entered = 0;
    sb->broken = false;
    sb->mode = 0;
    *out = sb;
    return SDV2_OK;
}

int32_t sdv2_stream_batch_destroy(sdv2_stream_batch* sb) {
    delete sb;
    return SDV2_OK;
}

int32_t sdv2_stream_batch_reset(sdv2_stream_batch* sb) {
    if (!sb) return fail(SDV2_INVALID_ARG, "handle is null");
    for (int r = 0; r < SDV2_MAX_BATCH; ++r) sb->depth[r] = -1;
    sb->entered = 0;
    sb->broken = false;
    sb->mode = 0;
    return SDV2_OK;
}

}  // extern "C"

namespace {
// One micro-step of the rotation for either kind of row.  io == nullptr: rows are hidden states [L, C] and level[d] is
// the timestep of depth d.  Otherwise rows are latents [16, F, 2 grid_h, 2 grid_w], level[0 .. n] are the noise levels
// (the row at depth d goes from level[d] to level[d + 1]) and eps_by_depth_dev[d] is the noise mixed into the row at
// depth d at its new level; eps_rows_dev is workspace for the same noise in row order.
int32_t stream_batch_step_impl(sdv2_stream_batch* sb, const sdv2_model_cfg* cfg, const sdv2_model_weights* mw,
                               const sdv2_io_weights* io, sdv2_kv_cache* cache, const float* in_dev, int32_t frame_pos0,
                               const float* level, const float* eps_by_depth_dev, float* eps_rows_dev,
                               const void* const* kt_dev, const void* const* vtt_dev, float* out_dev,
                               int32_t* emitted_out, int32_t* rows_out, void* workspace_dev, size_t workspace_bytes,
                               void* hip_stream) {
    const int n = sb->n_steps;
    const int L = sb->n_frames * cfg->grid_h * cfg->grid_w;
    const size_t row_floats = io ? (size_t)4 * kLatentChannels * L : sb->row_floats;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const size_t row_bytes = row_floats * sizeof(float);

    // the entering chunk takes the row that the chunk emitted n micro-steps after it entered has left
    int new_row = -1;
    if (in_dev) {
        new_row = (int)(sb->entered % n);
        if (sb->depth[new_row] >= 0) return fail(SDV2_BAD_STATE, "row %d is still occupied", new_row);
        HIP_TRY(hipMemcpyAsync(sb->x_pipe + (size_t)new_row * row_floats, in_dev, row_bytes, hipMemcpyDeviceToDevice, s),
                "copy of the entering chunk");
        sb->depth[new_row] = 0;
        sb->frame_pos0[new_row] = frame_pos0;
        sb->entered += 1;
    }
    // one batched denoising step per run of occupied rows that is contiguous in memory: one run in steady state and
    // while the pipeline fills, at most two while it drains
    int rows = 0;
    std::vector<const void*> kt, vtt;
    int r = 0;
    while (r < n) {
        if (sb->depth[r] < 0) {
            ++r;
            continue;
        }
        int r1 = r;
        while (r1 < n && sb->depth[r1] >= 0) ++r1;
        const int B = r1 - r;
        sdv2_chunk_desc descs[SDV2_MAX_BATCH];
        float lv[SDV2_MAX_BATCH], lv_next[SDV2_MAX_BATCH];
        bool need_eps = false;
        for (int b = 0; b < B; ++b) {
            const int d = sb->depth[r + b];
            descs[b].stream_id = sb->cache_ids[d];
            descs[b].frame_pos0 = sb->frame_pos0[r + b];
            descs[b].n_frames = sb->n_frames;
            descs[b].advance = 1;
            lv[b] = level[d];
            lv_next[b] = io ? level[d + 1] : 0.0f;
            need_eps = need_eps || lv_next[b] > 0.0f;
        }
        kt.assign((size_t)cfg->n_layers * B, nullptr);
        vtt.assign((size_t)cfg->n_layers * B, nullptr);
        for (int layer = 0; layer < cfg->n_layers; ++layer)
            for (int b = 0; b < B; ++b) {
                kt[(size_t)layer * B + b] = kt_dev[layer];
                vtt[(size_t)layer * B + b] = vtt_dev[layer];
            }
        int32_t rc = SDV2_OK;
        float* rows_ptr = sb->x_pipe + (size_t)r * row_floats;
        if (!io) {
            rc = sdv2_denoise_step(cfg, mw, cache, rows_ptr, lv, nullptr, kt.data(), vtt.data(), descs, B, workspace_dev,
                                   workspace_bytes, hip_stream);
        } else {
            if (need_eps) {                           // the noise of each depth, in the order of the rows of this run
                for (int b = 0; b < B; ++b) {
                    if (!(lv_next[b] > 0.0f)) continue;
                    const hipError_t e = hipMemcpyAsync(eps_rows_dev + (size_t)b * row_floats,
                                                        eps_by_depth_dev + (size_t)sb->depth[r + b] * row_floats, row_bytes,
                                                        hipMemcpyDeviceToDevice, s);
                    if (e != hipSuccess) {
                        rc = fail(SDV2_HIP_ERROR, "copy of the noise of depth %d: %s", sb->depth[r + b], hipGetErrorString(e));
                        break;
                    }
                }
            }
            if (!rc)
                rc = sdv2_denoise_latents_step(cfg, mw, io, cache, rows_ptr, need_eps ? eps_rows_dev : nullptr, nullptr, lv, lv_next,
                                               kt.data(), vtt.data(), descs, B, workspace_dev, workspace_bytes, hip_stream);
        }
        if (rc) {
            if (rows == 0 && new_row >= 0) {          // nothing has run: take the entering chunk out again
                sb->depth[new_row] = -1;
                sb->entered -= 1;
            } else if (rows > 0) {
                sb->broken = true;
            }
            return rc;
        }
        for (int b = 0; b < B; ++b) sb->depth[r + b] += 1;
        rows += B;
        r = r1;
    }
    *emitted_out = 0;
    for (int row = 0; row < n; ++row) {
        if (sb->depth[row] == n) {                    // finished its last step: the clean latent of this micro-step
            HIP_TRY(hipMemcpyAsync(out_dev, sb->x_pipe + (size_t)row * row_floats, row_bytes, hipMemcpyDeviceToDevice, s),
                    "copy of the finished chunk");
            sb->depth[row] = -1;
            *emitted_out = 1;
        }
    }
    if (rows_out) *rows_out = rows;
    return SDV2_OK;
}

// the checks the two kinds of step share; returns 0 or the error
int32_t stream_batch_check(sdv2_stream_batch* sb, const sdv2_model_cfg* cfg, const sdv2_model_weights* mw, sdv2_kv_cache* cache,
                           const float* in_dev, int32_t frame_pos0, const void* const* kt_dev, const void* const* vtt_dev,
                           int mode) {
    if (!sb) return fail(SDV2_INVALID_ARG, "handle is null");
    if (sb->broken) return fail(SDV2_BAD_STATE, "an earlier micro-step failed half way: reset the pipeline and the caches");
    if (sb->mode != 0 && sb->mode != mode)
        return fail(SDV2_BAD_STATE, "the pipeline holds %s: reset it before stepping it with the other kind of row",
                    sb->mode == 1 ? "hidden states" : "latents");
    const char* why;
    if (!model_cfg_ok(cfg, &why)) return fail(SDV2_INVALID_ARG, "%s", why);
    if (!mw || !cache || !kt_dev || !vtt_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    if ((size_t)sb->n_frames * cfg->grid_h * cfg->grid_w * cfg->C != sb->row_floats)
        return fail(SDV2_INVALID_ARG, "cfg differs from the one the pipeline was created with");
    if (in_dev && frame_pos0 < 0) return fail(SDV2_INVALID_ARG, "frame_pos0 < 0");
    for (int d = 0; d < sb->n_steps; ++d)
        if (sb->cache_ids[d] >= cache->cfg.n_streams) return fail(SDV2_INVALID_ARG, "cache stream %d of depth %d out of range", sb->cache_ids[d], d);
    for (int layer = 0; layer < cfg->n_layers; ++layer)
        if (!kt_dev[layer] || !vtt_dev[layer]) return fail(SDV2_INVALID_ARG, "text K/V of layer %d is null", layer);
    return SDV2_OK;
}
}  // namespace

extern "C" {

int32_t sdv2_stream_batch_step(sdv2_stream_batch* sb, const sdv2_model_cfg* cfg, const sdv2_model_weights* mw,
                               sdv2_kv_cache* cache, const float* x_in_dev, int32_t frame_pos0,
                               const float* timesteps_host, const void* const* kt_dev, const void* const* vtt_dev,
                               float* x_out_dev, int32_t* emitted_out, int32_t* rows_out, void* workspace_dev,
                               size_t workspace_bytes, void* hip_stream) {
    const int32_t bad = stream_batch_check(sb, cfg, mw, cache, x_in_dev, frame_pos0, kt_dev, vtt_dev, 1);
    if (bad) return bad;
    if (!timesteps_host || !x_out_dev || !emitted_out || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    const int L = sb->n_frames * cfg->grid_h * cfg->grid_w;
    const size_t need = sdv2_denoise_workspace_bytes(cfg, sb->n_steps, L);
    if (workspace_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, need);
    const int32_t rc = stream_batch_step_impl(sb, cfg, mw, nullptr, cache, x_in_dev, frame_pos0, timesteps_host, nullptr, nullptr,
                                              kt_dev, vtt_dev, x_out_dev, emitted_out, rows_out, workspace_dev, workspace_bytes,
                                              hip_stream);
    if (!rc) sb->mode = 1;
    return rc;
}

size_t sdv2_stream_batch_latents_workspace_bytes(const sdv2_model_cfg* cfg, int32_t n_steps, int32_t n_frames) {
    const char* why;
    if (!model_cfg_ok(cfg, &why) || n_steps < 1 || n_steps > SDV2_MAX_BATCH || n_frames < 1) {
        fail(SDV2_INVALID_ARG, "bad cfg, n_steps or n_frames");
        return 0;
    }
    const int L = n_frames * cfg->grid_h * cfg->grid_w;
    const size_t step = sdv2_denoise_latents_workspace_bytes(cfg, n_steps, L);
    if (!step) return 0;
    return step + align_up((size_t)n_steps * 4 * kLatentChannels * L * sizeof(float), 256);
}

int32_t sdv2_stream_batch_latents_step(sdv2_stream_batch* sb, const sdv2_model_cfg* cfg, const sdv2_model_weights* mw,
                                       const sdv2_io_weights* io, sdv2_kv_cache* cache, const float* z_in_dev,
                                       int32_t frame_pos0, const float* sigmas_host, const float* eps_by_depth_dev,
                                       const void* const* kt_dev, const void* const* vtt_dev, float* z_out_dev,
                                       int32_t* emitted_out, int32_t* rows_out, void* workspace_dev, size_t workspace_bytes,
                                       void* hip_stream) {
    const int32_t bad = stream_batch_check(sb, cfg, mw, cache, z_in_dev, frame_pos0, kt_dev, vtt_dev, 2);
    if (bad) return bad;
    if (!io_weights_ok(io)) return fail(SDV2_INVALID_ARG, "bad io weights");
    if (!sigmas_host || !z_out_dev || !emitted_out || !workspace_dev) return fail(SDV2_INVALID_ARG, "null pointer");
    const int n = sb->n_steps;
    bool any_noise = false;
    for (int d = 0; d <= n; ++d) {
        const float sg = sigmas_host[d];
        if (!(sg >= 0.0f && sg <= 1.0f) || (d < n && !(sg > 0.0f)) || (d > 0 && !(sg <= sigmas_host[d - 1])))
            return fail(SDV2_INVALID_ARG, "noise levels must fall from at most 1 to at least 0, all but the last above 0 (level %d)", d);
        any_noise = any_noise || (d > 0 && sg > 0.0f);
    }
    if (any_noise && !eps_by_depth_dev) return fail(SDV2_INVALID_ARG, "a level after the first is above 0 but eps_by_depth_dev is null");
    const size_t need = sdv2_stream_batch_latents_workspace_bytes(cfg, n, sb->n_frames);
    if (!need || workspace_bytes < need) return fail(SDV2_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, need);
    const int L = sb->n_frames * cfg->grid_h * cfg->grid_w;
    const size_t step_ws = sdv2_denoise_latents_workspace_bytes(cfg, n, L);
    float* eps_rows = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace_dev) + step_ws);
    const int32_t rc = stream_batch_step_impl(sb, cfg, mw, io, cache, z_in_dev, frame_pos0, sigmas_host, eps_by_depth_dev, eps_rows,
                                              kt_dev, vtt_dev, z_out_dev, emitted_out, rows_out, workspace_dev, step_ws, hip_stream);
    if (!rc) sb->mode = 2;
    return rc;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------ profiling helpers
extern "C" {

int32_t sdv2_prof_peak_mfma(int32_t iters, int32_t workgroups, float* sink_dev, size_t sink_floats, double* flops_out,
                            void* hip_stream) {
    if (iters <= 0 || workgroups <= 0 || workgroups > 65536) return fail(SDV2_INVALID_ARG, "iters and workgroups must be positive");
    if (!sink_dev || sink_floats < (size_t)workgroups * 512)
        return fail(SDV2_INVALID_ARG, "sink needs %zu floats", (size_t)workgroups * 512);
    HIP_TRY(launch_peak_mfma(iters, workgroups, sink_dev, static_cast<hipStream_t>(hip_stream)), "peak mfma kernel");
    if (flops_out) *flops_out = peak_mfma_flops(iters, workgroups);
    return SDV2_OK;
}

int32_t sdv2_prof_peak_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream) {
    if (!src_dev || !dst_dev || bytes == 0 || bytes % 16) return fail(SDV2_INVALID_ARG, "null pointer, or bytes not a positive multiple of 16");
    if (reinterpret_cast<uintptr_t>(src_dev) % 16 || reinterpret_cast<uintptr_t>(dst_dev) % 16)
        return fail(SDV2_INVALID_ARG, "buffers must be 16-byte aligned");
    HIP_TRY(launch_peak_copy(src_dev, dst_dev, bytes, static_cast<hipStream_t>(hip_stream)), "peak copy kernel");
    return SDV2_OK;
}

int32_t sdv2_prof_lds_rates(int32_t iters, void* scratch_dev, size_t scratch_bytes, void* hip_stream) {
    if (iters <= 0 || iters > (1 << 20)) return fail(SDV2_INVALID_ARG, "iters = %d out of range", iters);
    if (!scratch_dev || scratch_bytes < 40960) return fail(SDV2_INVALID_ARG, "scratch is null or below 40960 bytes");
    if (reinterpret_cast<uintptr_t>(scratch_dev) % 256) return fail(SDV2_INVALID_ARG, "scratch must be 256-byte aligned");
    unsigned char* p = static_cast<unsigned char*>(scratch_dev);
    // [0, 32) three tick counts; [2048, 4096) sink; [8192, 40960) the 32 KB the direct loads read
    HIP_TRY(launch_peak_lds(iters, p + 8192, reinterpret_cast<float*>(p + 2048), reinterpret_cast<unsigned long long*>(p),
                            static_cast<hipStream_t>(hip_stream)), "LDS rate kernels");
    return SDV2_OK;
}

int32_t sdv2_prof_kernel_name(int32_t kind, int32_t B, int32_t L, int32_t a0, int32_t a1, int32_t a2, char* out,
                              size_t capacity) {
    if (!out || capacity < 8) return fail(SDV2_INVALID_ARG, "out is null or too small");
    if (kind == 0) {                                   // GEMM: rows = B * L, a0 = N, a1 = K, a2 = epilogue
        if (B <= 0 || L <= 0 || a0 <= 0 || a1 <= 0 || a2 < 0 || a2 > 3) return fail(SDV2_INVALID_ARG, "bad GEMM shape");
        gemm_plan_name(B * L, a0, a1, a2, out, capacity);
        return SDV2_OK;
    }
    if (kind == 1) {                                   // attention: a0 = heads, a1 = keys, a2 = capacity in slots
        if (B <= 0 || B > SDV2_MAX_BATCH || L <= 0 || a0 <= 0 || a1 <= 0 || a2 < a1) return fail(SDV2_INVALID_ARG, "bad attention shape");
        AttnArgs a;
        memset(&a, 0, sizeof(a));
        a.B = B;
        a.L = L;
        a.H = a0;
        for (int b = 0; b < B; ++b) {
            a.kv_len[b] = a1;
            a.cap[b] = a2;
        }
        attention_plan_name(a, out, capacity);
        return SDV2_OK;
    }
    return fail(SDV2_INVALID_ARG, "kind must be 0 (GEMM) or 1 (attention)");
}

int32_t sdv2_prof_begin(int32_t max_samples) {
    if (max_samples <= 0 || max_samples > (1 << 20)) return fail(SDV2_INVALID_ARG, "max_samples out of range");
    if (g_prof.on) return fail(SDV2_BAD_STATE, "profiling already on");
    g_prof.start.resize(max_samples);
    g_prof.stop.resize(max_samples);
    g_prof.tag.assign(max_samples, -1);
    for (int i = 0; i < max_samples; ++i) {
        HIP_TRY(hipEventCreate(&g_prof.start[i]), "event create");
        HIP_TRY(hipEventCreate(&g_prof.stop[i]), "event create");
    }
    g_prof.n = 0;
    g_prof.on = true;
    return SDV2_OK;
}

int32_t sdv2_prof_end(int32_t* tags_out, float* ms_out, int32_t capacity, int32_t* n_out) {
    if (!g_prof.on) return fail(SDV2_BAD_STATE, "profiling is not on");
    if (!tags_out || !ms_out || !n_out) return fail(SDV2_INVALID_ARG, "null pointer");
    g_prof.on = false;
    int32_t rc = SDV2_OK;
    const int n = g_prof.n < capacity ? g_prof.n : capacity;
    for (int i = 0; i < n && rc == SDV2_OK; ++i) {
        hipError_t e = hipEventSynchronize(g_prof.stop[i]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms_out[i], g_prof.start[i], g_prof.stop[i]);
        if (e != hipSuccess) rc = hip_fail(e, "event elapsed");
        tags_out[i] = g_prof.tag[i];
    }
    *n_out = n;
    for (size_t i = 0; i < g_prof.start.size(); ++i) {
        hipEventDestroy(g_prof.start[i]);
        hipEventDestroy(g_prof.stop[i]);
    }
    g_prof.start.clear();
    g_prof.stop.clear();
    g_prof.n = 0;
    return rc;
}

}  // extern "C"
