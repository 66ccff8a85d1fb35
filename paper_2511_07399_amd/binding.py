"""ctypes binding of libsdv2: argument marshalling only.

Every function has the name of the C entry point without the ``sdv2_`` prefix
and passes torch device pointers straight through; no step of the block runs
in Python or in torch.  torch is used for device memory and for the current
HIP stream.  If the library has not been built, loading raises.
"""

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdv2.so")
MAX_BATCH = 8
HEAD_DIM = 128

OK, INVALID_ARG, BAD_STATE, WORKSPACE_TOO_SMALL, HIP_ERROR = 0, -1, -2, -3, -4


class Sdv2Error(RuntimeError):
    def __init__(self, code, text):
        super().__init__("sdv2 error %d: %s" % (code, text))
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("C", C.c_int32), ("n_heads", C.c_int32), ("ffn_dim", C.c_int32),
                ("grid_h", C.c_int32), ("grid_w", C.c_int32), ("text_len", C.c_int32), ("n_layers", C.c_int32),
                ("t_dim", C.c_int32), ("eps", C.c_float), ("rope_base", C.c_float)]


class CacheCfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("n_layers", C.c_int32), ("n_streams", C.c_int32),
                ("n_heads", C.c_int32), ("tokens_per_frame", C.c_int32), ("sink_tokens", C.c_int32),
                ("window_tokens", C.c_int32)]


_BLOCK_FIELDS = ("W_qkv", "b_qkv", "g_q", "g_k", "W_o", "b_o", "mod_table", "ln3_gamma", "ln3_beta", "W_cq", "b_cq",
                 "g_cq", "W_ck", "b_ck", "g_ck", "W_cv", "b_cv", "W_co", "b_co", "W_1", "b_1", "W_2", "b_2")


class BlockWeights(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("reserved", C.c_uint32)] + [(n, C.c_void_p) for n in _BLOCK_FIELDS]


class ModelWeights(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("reserved", C.c_uint32), ("blocks", C.POINTER(BlockWeights)),
                ("W_t1", C.c_void_p), ("b_t1", C.c_void_p), ("W_t2", C.c_void_p), ("b_t2", C.c_void_p),
                ("W_mod", C.c_void_p), ("b_mod", C.c_void_p)]


class ChunkDesc(C.Structure):
    _fields_ = [("stream_id", C.c_int32), ("frame_pos0", C.c_int32), ("n_frames", C.c_int32), ("advance", C.c_int32)]


class CacheState(C.Structure):
    _fields_ = [("total", C.c_int64), ("evicted", C.c_int64), ("sink_fill", C.c_int32), ("win_fill", C.c_int32),
                ("oldest_slot", C.c_int32), ("next_slot", C.c_int32)]


class IoWeights(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("reserved", C.c_uint32), ("W_pe", C.c_void_p), ("b_pe", C.c_void_p),
                ("head_table", C.c_void_p), ("W_head", C.c_void_p), ("b_head", C.c_void_p)]


class MotionCfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("k", C.c_int32), ("sigma", C.c_float), ("lam", C.c_float),
                ("s_min", C.c_float), ("s_max", C.c_float), ("s_init", C.c_float)]


EXPORTS = (
    "sdv2_last_error", "sdv2_version", "sdv2_kv_cache_bytes", "sdv2_kv_cache_init", "sdv2_kv_cache_destroy",
    "sdv2_kv_cache_reset", "sdv2_kv_cache_append_evict", "sdv2_kv_cache_state", "sdv2_kv_cache_slot_map",
    "sdv2_kv_cache_device_ptrs", "sdv2_sink_similarity_workspace_bytes", "sdv2_sink_similarity",
    "sdv2_kv_cache_refresh_sink", "sdv2_kv_cache_rotate_keys", "sdv2_motion_state_bytes", "sdv2_motion_init",
    "sdv2_motion_update", "sdv2_slo_pick_batch", "sdv2_text_kv_bytes", "sdv2_text_kv_workspace_bytes", "sdv2_text_kv_prepare",
    "sdv2_conditioning_workspace_bytes", "sdv2_conditioning", "sdv2_block_workspace_bytes",
    "sdv2_dit_block_forward", "sdv2_denoise_workspace_bytes", "sdv2_denoise_step", "sdv2_gemm_workspace_bytes", "sdv2_gemm_bf16",
    "sdv2_attention_workspace_bytes", "sdv2_attention_bf16", "sdv2_prof_begin", "sdv2_prof_end",
    "sdv2_prof_peak_mfma", "sdv2_prof_peak_copy", "sdv2_prof_lds_rates", "sdv2_prof_kernel_name", "sdv2_tuning_set", "sdv2_gemm_noalloc_max_scratch_bytes",
    "sdv2_gemm_bf16_noalloc", "sdv2_stream_batch_rows_bytes", "sdv2_stream_batch_create", "sdv2_stream_batch_destroy",
    "sdv2_stream_batch_reset", "sdv2_stream_batch_step", "sdv2_denoise_graph_state_bytes", "sdv2_denoise_graph_create",
    "sdv2_denoise_graph_launch", "sdv2_denoise_graph_destroy", "sdv2_timestep_vector", "sdv2_latent_io_workspace_bytes",
    "sdv2_patch_embed", "sdv2_output_head", "sdv2_noise_latents", "sdv2_sampler_update",
    "sdv2_denoise_latents_workspace_bytes", "sdv2_denoise_latents_step", "sdv2_stream_batch_latents_workspace_bytes",
    "sdv2_stream_batch_latents_step",
)

LAUNCH_TAGS = ("adaLN-1", "QKV gemm", "rope+append", "self-attn", "out-proj gemm", "LN-3", "cross-q gemm",
               "cross-q norm", "cross-attn", "cross-out gemm", "adaLN-2", "FFN-1 gemm", "FFN-2 gemm", "k-split reduce",
               "split-KV merge")

_lib = None


def load_library():
    """Load libsdv2.so and declare the signatures.  Raises if it is missing or a symbol is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libsdv2.so is not built (%s); run `python __graft_entry__.py`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        getattr(lib, name)
    vp, i32, sz, f32p = C.c_void_p, C.c_int32, C.c_size_t, C.c_void_p
    lib.sdv2_last_error.restype = C.c_char_p
    lib.sdv2_version.restype = i32
    lib.sdv2_kv_cache_bytes.restype = sz
    lib.sdv2_kv_cache_bytes.argtypes = [C.POINTER(CacheCfg)]
    lib.sdv2_kv_cache_init.argtypes = [C.POINTER(CacheCfg), vp, sz, C.POINTER(vp)]
    lib.sdv2_kv_cache_destroy.argtypes = [vp]
    lib.sdv2_kv_cache_reset.argtypes = [vp, i32]
    lib.sdv2_kv_cache_append_evict.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp]
    lib.sdv2_kv_cache_state.argtypes = [vp, i32, i32, C.POINTER(CacheState)]
    lib.sdv2_kv_cache_slot_map.argtypes = [vp, i32, i32, C.POINTER(C.c_int64)]
    lib.sdv2_kv_cache_device_ptrs.argtypes = [vp, i32, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                              C.POINTER(i32)]
    lib.sdv2_sink_similarity_workspace_bytes.restype = sz
    lib.sdv2_sink_similarity_workspace_bytes.argtypes = [vp]
    lib.sdv2_sink_similarity.argtypes = [vp, i32, i32, i32, vp, vp, sz, vp]
    lib.sdv2_kv_cache_refresh_sink.argtypes = [vp, i32, i32, i32, i32, vp]
    lib.sdv2_kv_cache_rotate_keys.argtypes = [vp, i32, i32, i32, C.c_float, vp]
    lib.sdv2_motion_state_bytes.restype = sz
    lib.sdv2_motion_state_bytes.argtypes = [C.POINTER(MotionCfg)]
    lib.sdv2_motion_init.argtypes = [C.POINTER(MotionCfg), vp, sz, vp]
    lib.sdv2_motion_update.argtypes = [C.POINTER(MotionCfg), vp, sz, vp, vp, i32, C.c_int64, vp, vp, vp, vp]
    lib.sdv2_slo_pick_batch.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_double), i32, i32, C.c_double, C.c_int64,
                                        C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.sdv2_text_kv_bytes.restype = sz
    lib.sdv2_text_kv_bytes.argtypes = [C.POINTER(ModelCfg)]
    lib.sdv2_text_kv_workspace_bytes.restype = sz
    lib.sdv2_text_kv_workspace_bytes.argtypes = [C.POINTER(ModelCfg)]
    lib.sdv2_text_kv_prepare.argtypes = [C.POINTER(ModelCfg), C.POINTER(BlockWeights), vp, vp, vp, vp, sz, vp]
    lib.sdv2_conditioning_workspace_bytes.restype = sz
    lib.sdv2_conditioning_workspace_bytes.argtypes = [C.POINTER(ModelCfg), i32]
    lib.sdv2_conditioning.argtypes = [C.POINTER(ModelCfg), C.POINTER(ModelWeights), i32, C.POINTER(C.c_float), f32p,
                                      f32p, vp, sz, vp]
    lib.sdv2_block_workspace_bytes.restype = sz
    lib.sdv2_block_workspace_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.sdv2_dit_block_forward.argtypes = [C.POINTER(ModelCfg), C.POINTER(BlockWeights), vp, i32, f32p, f32p,
                                           C.POINTER(vp), C.POINTER(vp), C.POINTER(ChunkDesc), i32, vp, sz, vp]
    lib.sdv2_denoise_workspace_bytes.restype = sz
    lib.sdv2_denoise_workspace_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.sdv2_denoise_step.argtypes = [C.POINTER(ModelCfg), C.POINTER(ModelWeights), vp, f32p, C.POINTER(C.c_float),
                                      f32p, C.POINTER(vp), C.POINTER(vp), C.POINTER(ChunkDesc), i32, vp, sz, vp]
    lib.sdv2_gemm_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.sdv2_gemm_workspace_bytes.restype = sz
    lib.sdv2_gemm_bf16.argtypes = [vp, vp, f32p, vp, i32, i32, i32, i32, f32p, f32p, i32, i32, vp, sz, vp]
    lib.sdv2_attention_workspace_bytes.restype = sz
    lib.sdv2_attention_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.sdv2_attention_bf16.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(i32), C.POINTER(i32), vp, i32,
                                        i32, i32, vp, sz, vp]
    lib.sdv2_prof_begin.argtypes = [i32]
    lib.sdv2_prof_end.argtypes = [C.POINTER(i32), C.POINTER(C.c_float), i32, C.POINTER(i32)]
    lib.sdv2_prof_peak_mfma.argtypes = [i32, i32, f32p, sz, C.POINTER(C.c_double), vp]
    lib.sdv2_prof_peak_copy.argtypes = [vp, vp, sz, vp]
    lib.sdv2_prof_lds_rates.argtypes = [i32, vp, sz, vp]
    lib.sdv2_tuning_set.argtypes = [C.c_char_p, C.c_char_p]
    lib.sdv2_prof_kernel_name.argtypes = [i32, i32, i32, i32, i32, i32, C.c_char_p, sz]
    lib.sdv2_gemm_noalloc_max_scratch_bytes.restype = sz
    lib.sdv2_denoise_graph_state_bytes.restype = sz
    lib.sdv2_denoise_graph_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(ModelWeights), vp, f32p, C.POINTER(vp),
                                              C.POINTER(vp), C.POINTER(i32), i32, i32, vp, sz, vp, sz, C.POINTER(vp)]
    lib.sdv2_denoise_graph_launch.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(ChunkDesc), i32, vp]
    lib.sdv2_denoise_graph_destroy.argtypes = [vp]
    lib.sdv2_stream_batch_rows_bytes.restype = sz
    lib.sdv2_stream_batch_rows_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.sdv2_stream_batch_create.argtypes = [C.POINTER(ModelCfg), i32, C.POINTER(i32), i32, f32p, sz, C.POINTER(vp)]
    lib.sdv2_stream_batch_destroy.argtypes = [vp]
    lib.sdv2_stream_batch_reset.argtypes = [vp]
    lib.sdv2_stream_batch_step.argtypes = [vp, C.POINTER(ModelCfg), C.POINTER(ModelWeights), vp, f32p, i32,
                                           C.POINTER(C.c_float), C.POINTER(vp), C.POINTER(vp), f32p, C.POINTER(i32),
                                           C.POINTER(i32), vp, sz, vp]
    lib.sdv2_gemm_bf16_noalloc.argtypes = [vp, vp, f32p, vp, i32, i32, i32, i32, f32p, f32p, i32, i32, vp]
    fp = C.POINTER(C.c_float)
    lib.sdv2_timestep_vector.argtypes = [C.POINTER(ModelCfg), C.POINTER(ModelWeights), i32, fp, f32p, vp, sz, vp]
    lib.sdv2_latent_io_workspace_bytes.restype = sz
    lib.sdv2_latent_io_workspace_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.sdv2_patch_embed.argtypes = [C.POINTER(ModelCfg), C.POINTER(IoWeights), f32p, i32, i32, f32p, vp, sz, vp]
    lib.sdv2_output_head.argtypes = [C.POINTER(ModelCfg), C.POINTER(IoWeights), f32p, f32p, i32, i32, f32p, vp, sz, vp]
    lib.sdv2_noise_latents.argtypes = [f32p, f32p, f32p, i32, C.c_int64, fp, vp]
    lib.sdv2_sampler_update.argtypes = [f32p, f32p, f32p, f32p, f32p, i32, C.c_int64, fp, fp, vp]
    lib.sdv2_denoise_latents_workspace_bytes.restype = sz
    lib.sdv2_denoise_latents_workspace_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.sdv2_denoise_latents_step.argtypes = [C.POINTER(ModelCfg), C.POINTER(ModelWeights), C.POINTER(IoWeights), vp,
                                              f32p, f32p, f32p, fp, fp, C.POINTER(vp), C.POINTER(vp),
                                              C.POINTER(ChunkDesc), i32, vp, sz, vp]
    lib.sdv2_stream_batch_latents_workspace_bytes.restype = sz
    lib.sdv2_stream_batch_latents_workspace_bytes.argtypes = [C.POINTER(ModelCfg), i32, i32]
    lib.sdv2_stream_batch_latents_step.argtypes = [vp, C.POINTER(ModelCfg), C.POINTER(ModelWeights), C.POINTER(IoWeights), vp,
                                                   f32p, i32, fp, f32p, C.POINTER(vp), C.POINTER(vp), f32p,
                                                   C.POINTER(i32), C.POINTER(i32), vp, sz, vp]
    _lib = lib
    return lib


def _check(rc):
    if rc != OK:
        raise Sdv2Error(rc, _lib.sdv2_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), "expected a contiguous %s device tensor" % dtype
    return t


# ------------------------------------------------------------------------------------------ config helpers
def model_cfg(C_, n_heads, ffn_dim, grid_h, grid_w, text_len, n_layers, t_dim=256, eps=1e-6, rope_base=10000.0):
    return ModelCfg(C.sizeof(ModelCfg), C_, n_heads, ffn_dim, grid_h, grid_w, text_len, n_layers, t_dim, eps,
                    rope_base)


def cache_cfg(n_layers, n_streams, n_heads, tokens_per_frame, sink_tokens, window_tokens):
    return CacheCfg(C.sizeof(CacheCfg), n_layers, n_streams, n_heads, tokens_per_frame, sink_tokens, window_tokens)


def block_weights(tensors):
    """BlockWeights struct from a dict of device tensors (W_qkv / b_qkv already concatenated).
    The caller keeps the tensors alive."""
    bw = BlockWeights()
    bw.struct_size = C.sizeof(BlockWeights)
    for name in _BLOCK_FIELDS:
        t = tensors.get(name)
        if t is not None:
            _dev(t, torch.bfloat16 if name.startswith("W_") else torch.float32)
            setattr(bw, name, t.data_ptr())
    return bw


def model_weights(tensors, blocks):
    """ModelWeights struct; ``blocks`` is a ctypes array of BlockWeights that the caller keeps alive."""
    mw = ModelWeights()
    mw.struct_size = C.sizeof(ModelWeights)
    mw.blocks = C.cast(blocks, C.POINTER(BlockWeights))
    for name in ("W_t1", "b_t1", "W_t2", "b_t2", "W_mod", "b_mod"):
        t = tensors.get(name)
        if t is not None:
            _dev(t, torch.bfloat16 if name.startswith("W_") else torch.float32)
            setattr(mw, name, t.data_ptr())
    return mw


def chunk_descs(descs):
    arr = (ChunkDesc * len(descs))()
    for i, (stream_id, frame_pos0, n_frames, advance) in enumerate(descs):
        arr[i] = ChunkDesc(stream_id, frame_pos0, n_frames, int(advance))
    return arr


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


# ------------------------------------------------------------------------------------------ cache
def kv_cache_bytes(cfg):
    load_library()
    n = _lib.sdv2_kv_cache_bytes(C.byref(cfg))
    if n == 0:
        _check(INVALID_ARG)
    return n


def kv_cache_init(cfg, storage):
    """storage: a uint8 device tensor of at least kv_cache_bytes(cfg) bytes.  Returns the opaque handle."""
    load_library()
    h = C.c_void_p()
    _check(_lib.sdv2_kv_cache_init(C.byref(cfg), _ptr(storage), storage.numel() * storage.element_size(),
                                   C.byref(h)))
    return h


def kv_cache_destroy(handle):
    _check(_lib.sdv2_kv_cache_destroy(handle))


def kv_cache_reset(handle, stream_id):
    _check(_lib.sdv2_kv_cache_reset(handle, stream_id))


def kv_cache_append_evict(handle, layer, stream_id, k, v, advance=True):
    _dev(k, torch.bfloat16)
    _dev(v, torch.bfloat16)
    _check(_lib.sdv2_kv_cache_append_evict(handle, layer, stream_id, _ptr(k), _ptr(v), k.shape[0], int(advance),
                                           _stream()))


def sink_similarity_workspace_bytes(handle):
    return int(_lib.sdv2_sink_similarity_workspace_bytes(handle))


def sink_similarity(handle, layer, stream_id, alpha, workspace, frame_back=0):
    """alpha (device fp32 [sink frames]) <- cos(frame `frame_back` of the latest append, sink frame i)."""
    _dev(alpha, torch.float32)
    _check(_lib.sdv2_sink_similarity(handle, layer, stream_id, frame_back, _ptr(alpha), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))


def kv_cache_refresh_sink(handle, layer, stream_id, sink_frame, frame_back=0):
    _check(_lib.sdv2_kv_cache_refresh_sink(handle, layer, stream_id, sink_frame, frame_back, _stream()))


def kv_cache_rotate_keys(handle, layer, stream_id, delta_frames, rope_base=10000.0):
    _check(_lib.sdv2_kv_cache_rotate_keys(handle, layer, stream_id, delta_frames, rope_base, _stream()))


def motion_cfg(k, sigma, lam, s_min, s_max, s_init):
    c = MotionCfg()
    c.struct_size = C.sizeof(MotionCfg)
    c.k, c.sigma, c.lam, c.s_min, c.s_max, c.s_init = k, sigma, lam, s_min, s_max, s_init
    return c


def motion_state_bytes(cfg):
    return int(_lib.sdv2_motion_state_bytes(C.byref(cfg)))


def motion_init(cfg, state):
    _check(_lib.sdv2_motion_init(C.byref(cfg), _ptr(state), state.numel() * state.element_size(), _stream()))


def motion_update(cfg, state, frames, prev_frame, d_out, dhat_out, s_out):
    """frames: device fp32 [T, n]; prev_frame: device fp32 [n] or None; outputs device fp32 [T]."""
    _dev(frames, torch.float32)
    _check(_lib.sdv2_motion_update(C.byref(cfg), _ptr(state), state.numel() * state.element_size(), _ptr(frames),
                                   None if prev_frame is None else _ptr(prev_frame), frames.shape[0],
                                   frames.shape[1], _ptr(d_out), _ptr(dhat_out), _ptr(s_out), _stream()))


def slo_pick_batch(latency_s, frames_per_chunk, f_slo, frames_collected, knee_tol=0.0):
    """latency_s: dict batch size -> seconds.  Returns None or (B*, f(B*), meets_slo)."""
    sizes = list(latency_s)
    n = len(sizes)
    bs = (C.c_int32 * n)(*sizes)
    ls = (C.c_double * n)(*[latency_s[b] for b in sizes])
    b_out, f_out, ok = C.c_int32(), C.c_double(), C.c_int32()
    _check(_lib.sdv2_slo_pick_batch(bs, ls, n, frames_per_chunk, f_slo, frames_collected, knee_tol, C.byref(b_out),
                                    C.byref(f_out), C.byref(ok)))
    return None if b_out.value == 0 else (b_out.value, f_out.value, bool(ok.value))


def kv_cache_state(handle, layer, stream_id):
    st = CacheState()
    _check(_lib.sdv2_kv_cache_state(handle, layer, stream_id, C.byref(st)))
    return {"total": st.total, "sink_fill": st.sink_fill, "win_fill": st.win_fill, "oldest_slot": st.oldest_slot,
            "next_slot": st.next_slot, "evicted": st.evicted}


def kv_cache_slot_map(handle, layer, stream_id, n_slots):
    buf = (C.c_int64 * n_slots)()
    _check(_lib.sdv2_kv_cache_slot_map(handle, layer, stream_id, buf))
    return list(buf)


def vt_columns(n):
    """Column of the V^T cache rows that holds each of the slots 0 .. n-1 (the layout stated in sdv2.h)."""
    s = torch.arange(n)
    return (s & ~12) | ((s & 4) << 1) | ((s & 8) >> 1)


def kv_cache_device_ptrs(handle, layer, stream_id):
    k, vt, ids, cap = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_int32()
    _check(_lib.sdv2_kv_cache_device_ptrs(handle, layer, stream_id, C.byref(k), C.byref(vt), C.byref(ids),
                                          C.byref(cap)))
    return k.value, vt.value, ids.value, cap.value


# ------------------------------------------------------------------------------------------ text K/V, conditioning
def text_kv_bytes(cfg):
    load_library()
    return _lib.sdv2_text_kv_bytes(C.byref(cfg))


def text_kv_workspace_bytes(cfg):
    load_library()
    return _lib.sdv2_text_kv_workspace_bytes(C.byref(cfg))


def text_kv_prepare(cfg, bw, ctx, kt, vtt, workspace):
    _dev(ctx, torch.bfloat16)
    _check(_lib.sdv2_text_kv_prepare(C.byref(cfg), C.byref(bw), _ptr(ctx), _ptr(kt), _ptr(vtt), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))


def conditioning_workspace_bytes(cfg, B):
    load_library()
    return _lib.sdv2_conditioning_workspace_bytes(C.byref(cfg), B)


def _timesteps(timesteps):
    if timesteps is None:
        return None
    return (C.c_float * len(timesteps))(*[float(t) for t in timesteps])


def conditioning(cfg, mw, B, e0, workspace, timesteps=None, tvec=None):
    _dev(e0, torch.float32)
    if tvec is not None:
        _dev(tvec, torch.float32)
    _check(_lib.sdv2_conditioning(C.byref(cfg), C.byref(mw), B, _timesteps(timesteps), _ptr(tvec), _ptr(e0),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


# ------------------------------------------------------------------------------------------ block and step
def block_workspace_bytes(cfg, B, L):
    load_library()
    return _lib.sdv2_block_workspace_bytes(C.byref(cfg), B, L)


def denoise_workspace_bytes(cfg, B, L):
    load_library()
    return _lib.sdv2_denoise_workspace_bytes(C.byref(cfg), B, L)


def dit_block_forward(cfg, bw, cache, layer, x, e0, kt_list, vtt_list, chunks, workspace):
    _dev(x, torch.float32)
    _dev(e0, torch.float32)
    _check(_lib.sdv2_dit_block_forward(C.byref(cfg), C.byref(bw), cache, layer, _ptr(x), _ptr(e0),
                                       _ptr_array(kt_list), _ptr_array(vtt_list), chunks, len(chunks),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def denoise_step(cfg, mw, cache, x, kt_array, vtt_array, chunks, workspace, timesteps=None, tvec=None):
    """kt_array / vtt_array: ctypes c_void_p arrays [n_layers * B] (see ptr_array)."""
    _dev(x, torch.float32)
    if tvec is not None:
        _dev(tvec, torch.float32)
    _check(_lib.sdv2_denoise_step(C.byref(cfg), C.byref(mw), cache, _ptr(x), _timesteps(timesteps), _ptr(tvec),
                                  kt_array, vtt_array, chunks, len(chunks), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()))


ptr_array = _ptr_array


# ------------------------------------------------------------------------------------------ dense helpers
def gemm_workspace_bytes(M, N, K, epilogue):
    load_library()
    return int(_lib.sdv2_gemm_workspace_bytes(M, N, K, epilogue))


def gemm_bf16(a, w, bias, out, epilogue=0, gate_a=None, gate_b=None, gate_b_stride=0, rows_per_gate=1, workspace=None):
    load_library()
    _dev(a, torch.bfloat16)
    _dev(w, torch.bfloat16)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K and tuple(out.shape) == (M, N)
    _dev(out, torch.bfloat16 if epilogue in (0, 1) else torch.float32)
    _check(_lib.sdv2_gemm_bf16(_ptr(a), _ptr(w), _ptr(bias), _ptr(out), M, N, K, epilogue, _ptr(gate_a), _ptr(gate_b),
                               gate_b_stride, rows_per_gate, _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _stream()))


def gemm_noalloc_max_scratch_bytes():
    load_library()
    return int(_lib.sdv2_gemm_noalloc_max_scratch_bytes())


def gemm_bf16_noalloc(a, w, bias, out, epilogue=0, gate_a=None, gate_b=None, gate_b_stride=0, rows_per_gate=1):
    load_library()
    _dev(a, torch.bfloat16)
    _dev(w, torch.bfloat16)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K and tuple(out.shape) == (M, N)
    _dev(out, torch.bfloat16 if epilogue in (0, 1) else torch.float32)
    _check(_lib.sdv2_gemm_bf16_noalloc(_ptr(a), _ptr(w), _ptr(bias), _ptr(out), M, N, K, epilogue, _ptr(gate_a),
                                       _ptr(gate_b), gate_b_stride, rows_per_gate, _stream()))


def attention_workspace_bytes(B, L, C_, max_kv_len):
    load_library()
    return _lib.sdv2_attention_workspace_bytes(B, L, C_, max_kv_len)


def attention_bf16(q, k_list, vt_list, kv_lens, caps, o, n_heads, workspace):
    load_library()
    _dev(q, torch.bfloat16)
    _dev(o, torch.bfloat16)
    B, L, _ = q.shape
    kl = (C.c_int32 * B)(*kv_lens)
    cp = (C.c_int32 * B)(*caps)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib.sdv2_attention_bf16(_ptr(q), _ptr_array(k_list), _ptr_array(vt_list), kl, cp, _ptr(o), B, L, n_heads,
                                    _ptr(workspace), ws_bytes, _stream()))


# ------------------------------------------------------------------------------------------ profiling helpers
def prof_begin(max_samples):
    load_library()
    _check(_lib.sdv2_prof_begin(max_samples))


def prof_end(capacity):
    """Returns a list of (tag, milliseconds), one per bracketed launch, in launch order.  Blocks."""
    tags = (C.c_int32 * capacity)()
    ms = (C.c_float * capacity)()
    n = C.c_int32()
    _check(_lib.sdv2_prof_end(tags, ms, capacity, C.byref(n)))
    return [(tags[i], ms[i]) for i in range(n.value)]


def prof_peak_mfma(iters, workgroups, sink):
    """Enqueues the register-resident matrix-instruction loop; returns the flops of the launch."""
    load_library()
    _dev(sink, torch.float32)
    flops = C.c_double()
    _check(_lib.sdv2_prof_peak_mfma(iters, workgroups, _ptr(sink), sink.numel(), C.byref(flops), _stream()))
    return flops.value


def prof_peak_copy(src, dst):
    load_library()
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(_lib.sdv2_prof_peak_copy(_ptr(src), _ptr(dst), n, _stream()))
    return n


def prof_lds_rates(iters, scratch):
    """Enqueues the three LDS-rate launches; the three tick counts are the first three int64 of ``scratch``."""
    load_library()
    _check(_lib.sdv2_prof_lds_rates(iters, _ptr(scratch), scratch.numel() * scratch.element_size(), _stream()))


def prof_kernel_name(kind, B, L, a0, a1, a2):
    """kind "gemm": (N, K, epilogue) = (a0, a1, a2); kind "attention": (heads, keys, capacity) = (a0, a1, a2)."""
    load_library()
    buf = C.create_string_buffer(128)
    _check(_lib.sdv2_prof_kernel_name(0 if kind == "gemm" else 1, B, L, a0, a1, a2, buf, 128))
    return buf.value.decode()


def tuning_set(name, value=None):
    """Test / sweep hook: force a kernel plan ("gemm_tile", "attn_waves", "attn_splits"); None clears it."""
    load_library()
    _check(_lib.sdv2_tuning_set(name.encode(), None if value is None else str(value).encode()))


# ------------------------------------------------------------------------------------------ stream batch
def stream_batch_rows_bytes(cfg, n_steps, n_frames):
    load_library()
    return int(_lib.sdv2_stream_batch_rows_bytes(C.byref(cfg), n_steps, n_frames))


def stream_batch_create(cfg, n_steps, cache_stream_ids, n_frames, rows):
    """rows: uint8 device tensor of stream_batch_rows_bytes bytes that the caller keeps alive."""
    load_library()
    ids = (C.c_int32 * n_steps)(*cache_stream_ids)
    h = C.c_void_p()
    _check(_lib.sdv2_stream_batch_create(C.byref(cfg), n_steps, ids, n_frames, _ptr(rows),
                                         rows.numel() * rows.element_size(), C.byref(h)))
    return h


def stream_batch_destroy(h):
    _check(_lib.sdv2_stream_batch_destroy(h))


def stream_batch_reset(h):
    _check(_lib.sdv2_stream_batch_reset(h))


def stream_batch_step(h, cfg, mw, cache, x_in, frame_pos0, timesteps, kt, vtt, x_out, workspace):
    """kt / vtt: ctypes pointer arrays [n_layers].  Returns (emitted, rows)."""
    if x_in is not None:
        _dev(x_in, torch.float32)
    _dev(x_out, torch.float32)
    ts = (C.c_float * len(timesteps))(*timesteps)
    emitted, rows = C.c_int32(), C.c_int32()
    _check(_lib.sdv2_stream_batch_step(h, C.byref(cfg), C.byref(mw), cache, _ptr(x_in), frame_pos0, ts, kt, vtt,
                                       _ptr(x_out), C.byref(emitted), C.byref(rows), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()))
    return bool(emitted.value), rows.value


# ------------------------------------------------------------------------------------------ the step as a replayed graph
def denoise_graph_state_bytes():
    load_library()
    return int(_lib.sdv2_denoise_graph_state_bytes())


def denoise_graph_create(cfg, mw, cache, x, kt_array, vtt_array, stream_ids, n_frames, workspace, state):
    """x, workspace, state: device tensors the caller keeps alive; kt_array / vtt_array as for denoise_step."""
    load_library()
    _dev(x, torch.float32)
    ids = (C.c_int32 * len(stream_ids))(*stream_ids)
    h = C.c_void_p()
    _check(_lib.sdv2_denoise_graph_create(C.byref(cfg), C.byref(mw), cache, _ptr(x), kt_array, vtt_array, ids,
                                          len(stream_ids), n_frames, _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _ptr(state),
                                          state.numel() * state.element_size(), C.byref(h)))
    return h


def denoise_graph_launch(h, timesteps, chunks):
    ts = (C.c_float * len(timesteps))(*timesteps)
    _check(_lib.sdv2_denoise_graph_launch(h, ts, chunks, len(chunks), _stream()))


def denoise_graph_destroy(h):
    _check(_lib.sdv2_denoise_graph_destroy(h))


# ------------------------------------------------------------------------------------------ latents in, latents out
def io_weights(tensors):
    """IoWeights struct from a dict of device tensors; the caller keeps the tensors alive."""
    io = IoWeights()
    io.struct_size = C.sizeof(IoWeights)
    for name in ("W_pe", "b_pe", "head_table", "W_head", "b_head"):
        t = tensors[name]
        _dev(t, torch.bfloat16 if name.startswith("W_") else torch.float32)
        setattr(io, name, t.data_ptr())
    return io


def _nbytes(t):
    return t.numel() * t.element_size()


def timestep_vector(cfg, mw, timesteps, tvec, workspace):
    _dev(tvec, torch.float32)
    _check(_lib.sdv2_timestep_vector(C.byref(cfg), C.byref(mw), len(timesteps), _timesteps(timesteps), _ptr(tvec),
                                     _ptr(workspace), _nbytes(workspace), _stream()))


def latent_io_workspace_bytes(cfg, B, L):
    load_library()
    return int(_lib.sdv2_latent_io_workspace_bytes(C.byref(cfg), B, L))


def patch_embed(cfg, io, z, x, workspace):
    """z fp32 [B, 16, F, 2 grid_h, 2 grid_w] -> x fp32 [B, L, C]."""
    _dev(z, torch.float32)
    _dev(x, torch.float32)
    _check(_lib.sdv2_patch_embed(C.byref(cfg), C.byref(io), _ptr(z), z.shape[0], z.shape[2], _ptr(x), _ptr(workspace),
                                 _nbytes(workspace), _stream()))


def output_head(cfg, io, x, tvec, v, workspace):
    """x fp32 [B, L, C], tvec fp32 [B, C] -> v fp32 [B, 16, F, 2 grid_h, 2 grid_w]."""
    _dev(x, torch.float32)
    _dev(tvec, torch.float32)
    _dev(v, torch.float32)
    _check(_lib.sdv2_output_head(C.byref(cfg), C.byref(io), _ptr(x), _ptr(tvec), v.shape[0], v.shape[2], _ptr(v),
                                 _ptr(workspace), _nbytes(workspace), _stream()))


def noise_latents(x, eps, out, rates):
    for t in (x, eps, out):
        _dev(t, torch.float32)
    B = len(rates)
    _check(_lib.sdv2_noise_latents(_ptr(x), _ptr(eps), _ptr(out), B, x.numel() // B, _timesteps(rates), _stream()))


def sampler_update(z, v, eps_next, z_next, x0, sigmas, sigmas_next):
    for t in (z, v, z_next):
        _dev(t, torch.float32)
    B = len(sigmas)
    _check(_lib.sdv2_sampler_update(_ptr(z), _ptr(v), _ptr(eps_next), _ptr(z_next), _ptr(x0), B, z.numel() // B,
                                    _timesteps(sigmas), _timesteps(sigmas_next), _stream()))


def denoise_latents_workspace_bytes(cfg, B, L):
    load_library()
    return int(_lib.sdv2_denoise_latents_workspace_bytes(C.byref(cfg), B, L))


def denoise_latents_step(cfg, mw, io, cache, z, eps_next, x0, sigmas, sigmas_next, kt_array, vtt_array, chunks,
                         workspace):
    """z fp32 [B, 16, F, 2 grid_h, 2 grid_w], updated in place; x0 optional, same shape."""
    _dev(z, torch.float32)
    _check(_lib.sdv2_denoise_latents_step(C.byref(cfg), C.byref(mw), C.byref(io), cache, _ptr(z), _ptr(eps_next),
                                          _ptr(x0), _timesteps(sigmas), _timesteps(sigmas_next), kt_array, vtt_array,
                                          chunks, len(chunks), _ptr(workspace), _nbytes(workspace), _stream()))


def stream_batch_latents_workspace_bytes(cfg, n_steps, n_frames):
    load_library()
    return int(_lib.sdv2_stream_batch_latents_workspace_bytes(C.byref(cfg), n_steps, n_frames))


def stream_batch_latents_step(h, cfg, mw, io, cache, z_in, frame_pos0, sigmas, eps_by_depth, kt, vtt, z_out, workspace):
    """One micro-step with rows of latents; returns (emitted, rows).  z_in: fp32 latent of the entering chunk or None;
    sigmas: n_steps + 1 noise levels; eps_by_depth: fp32 [n_steps, 16, F, 2 grid_h, 2 grid_w] or None."""
    if z_in is not None:
        _dev(z_in, torch.float32)
    if eps_by_depth is not None:
        _dev(eps_by_depth, torch.float32)
    _dev(z_out, torch.float32)
    emitted, rows = C.c_int32(0), C.c_int32(0)
    _check(_lib.sdv2_stream_batch_latents_step(h, C.byref(cfg), C.byref(mw), C.byref(io), cache, _ptr(z_in), frame_pos0,
                                               _timesteps(sigmas), _ptr(eps_by_depth), kt, vtt, _ptr(z_out),
                                               C.byref(emitted), C.byref(rows), _ptr(workspace), _nbytes(workspace), _stream()))
    return bool(emitted.value), rows.value
