"""Oracle of the causal video-DiT block for one streaming chunk (TEST INFRASTRUCTURE ONLY).

The paper names the model (a causal DiT derived from Wan 2.1 and CausVid,
Section 5.1 "Models"), its precision (bf16, Section 5.1), the use of exact
flash-style attention (Section 4.1, SLO-aware batching scheduler) and its
per-layer cost (Appendix B: 24 b L_q C^2 flops of projections and FFN plus
4 b L_q L_kv C of attention), but prints no block equations.  The equations
below are this build's reading and are written out as the plain definition:
dense matrix products, a dense softmax over the explicit resident key set,
no tiling, no online softmax, no fusion.  ``numpy.matmul`` is the only library
primitive used.

Conventions
  * one stream at a time: ``x`` is ``[L, C]``; batches are a loop outside;
  * linear layers are ``y = x @ W.T + b`` with ``W`` stored ``[out, in]``;
  * head ``h`` owns columns ``[h*D, (h+1)*D)``;
  * modulation rows are (shift1, scale1, gate1, shift2, scale2, gate2).
"""

import math

import numpy as np

EPS = 1e-6
ROPE_BASE = 10000.0


# --------------------------------------------------------------------------- pointwise
def layer_norm(x, gamma=None, beta=None, eps=EPS):
    """Per-row (x - mean) / sqrt(var + eps), biased variance, optional affine."""
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mean) / np.sqrt(var + eps)
    if gamma is not None:
        y = y * gamma
    if beta is not None:
        y = y + beta
    return y


def rms_norm(x, gain, eps=EPS):
    """Per-row x / sqrt(mean(x^2) + eps) * gain, over the whole last axis (all heads)."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def gelu_tanh(x):
    """GELU, tanh form: x/2 * (1 + tanh(sqrt(2/pi) * (x + 0.044715 x^3)))."""
    c = math.sqrt(2.0 / math.pi)
    return 0.5 * x * (1.0 + np.tanh(c * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def linear(x, w, b):
    return np.matmul(x, w.T) + b


# --------------------------------------------------------------------------- RoPE
def rope_pair_split(head_dim):
    """How the D/2 rotation pairs of a head are shared out: (frame, row, col).

    Row and column each get floor(pairs/3); the frame axis gets the rest
    (22 | 21 | 21 for D = 128).
    """
    pairs = head_dim // 2
    third = pairs // 3
    return pairs - 2 * third, third, third


def token_positions(n_tokens, tokens_per_frame, grid_w, frame_pos0):
    """(frame, row, col) of each token of a chunk laid out frame-major, row-major."""
    i = np.arange(n_tokens)
    f = frame_pos0 + i // tokens_per_frame
    inside = i % tokens_per_frame
    return np.stack([f, inside // grid_w, inside % grid_w], axis=1)


def rope_3d(x, pos, dtype=np.float64):
    """Rotate ``x [L, H, D]`` by the 3-axis rotary embedding at ``pos [L, 3]``.

    Pair p of a head is the interleaved couple (x[2p], x[2p+1]).  Pairs are laid
    out [frame pairs | row pairs | col pairs]; pair j of an axis that owns d_a
    pairs turns by  pos_axis * 10000**(-j/d_a).
    """
    L, H, D = x.shape
    angles = []
    for axis, d_a in enumerate(rope_pair_split(D)):
        j = np.arange(d_a, dtype=np.float64)
        freq = ROPE_BASE ** (-j / d_a)
        angles.append(pos[:, axis:axis + 1].astype(np.float64) * freq[None, :])
    theta = np.concatenate(angles, axis=1).astype(dtype)        # [L, D/2]
    cos = np.cos(theta)[:, None, :]
    sin = np.sin(theta)[:, None, :]
    even = x[:, :, 0::2]
    odd = x[:, :, 1::2]
    out = np.empty_like(x)
    out[:, :, 0::2] = even * cos - odd * sin
    out[:, :, 1::2] = even * sin + odd * cos
    return out


# --------------------------------------------------------------------------- attention
def attention_dense(q, k, v, return_probs=False):
    """softmax(q k^T / sqrt(D)) v per head; q ``[Lq,H,D]``, k and v ``[Lk,H,D]``."""
    Lq, H, D = q.shape
    scores = np.matmul(q.transpose(1, 0, 2), k.transpose(1, 2, 0)) / math.sqrt(D)   # [H,Lq,Lk]
    scores = scores - scores.max(axis=-1, keepdims=True)
    e = np.exp(scores)
    probs = e / e.sum(axis=-1, keepdims=True)
    out = np.matmul(probs, v.transpose(1, 0, 2)).transpose(1, 0, 2)                # [Lq,H,D]
    if return_probs:
        return out, probs
    return out


def text_kv_prepare(ctx, w, dtype=np.float64):
    """Per prompt and layer: K_t = RMSNorm(ctx W_ck^T + b_ck) g_ck,  V_t = ctx W_cv^T + b_cv."""
    ctx = np.asarray(ctx, dtype=dtype)
    k_t = rms_norm(linear(ctx, w["W_ck"].astype(dtype), w["b_ck"].astype(dtype)), w["g_ck"].astype(dtype))
    v_t = linear(ctx, w["W_cv"].astype(dtype), w["b_cv"].astype(dtype))
    return k_t, v_t


# --------------------------------------------------------------------------- the block
def dit_block_forward(x, e0, w, cache, text_k, text_v, n_heads, tokens_per_frame, grid_w,
                      frame_pos0, advance=True, dtype=np.float64, debug=None):
    """One block on one chunk of one stream; returns the new ``x`` and updates ``cache``.

    x       [L, C]   hidden state of the chunk's tokens
    e0      [6, C]   timestep modulation shared by all layers
    w       dict of this layer's tensors (see module docstring for layouts)
    cache   oracle.kv_cache.RollingKVCache of this (layer, stream), width C
    text_k, text_v   [L_t, C] from text_kv_prepare
    frame_pos0       RoPE frame index of the chunk's first frame
    advance          True: new chunk (evicts); False: further denoising step of
                     the same chunk (overwrites the latest append)
    debug            optional dict that receives intermediates
    """
    f = lambda a: np.asarray(a, dtype=dtype)
    x = f(x)
    L, C = x.shape
    H = n_heads
    D = C // H
    mod = f(w["mod_table"]) + f(e0)
    shift1, scale1, gate1, shift2, scale2, gate2 = (mod[i] for i in range(6))

    # self-attention branch
    h = layer_norm(x) * (1.0 + scale1) + shift1
    q = rms_norm(linear(h, f(w["W_q"]), f(w["b_q"])), f(w["g_q"]))
    k = rms_norm(linear(h, f(w["W_k"]), f(w["b_k"])), f(w["g_k"]))
    v = linear(h, f(w["W_v"]), f(w["b_v"]))
    pos = token_positions(L, tokens_per_frame, grid_w, frame_pos0)
    q = rope_3d(q.reshape(L, H, D), pos, dtype)
    k = rope_3d(k.reshape(L, H, D), pos, dtype).reshape(L, C)
    cache.append_evict(k, v, advance=advance)
    k_res, v_res = cache.gather()                      # every resident token, this chunk included
    n_res = k_res.shape[0]
    attn = attention_dense(q, k_res.reshape(n_res, H, D), v_res.reshape(n_res, H, D)).reshape(L, C)
    upd_self = gate1 * linear(attn, f(w["W_o"]), f(w["b_o"]))
    x = x + upd_self

    # text cross-attention branch (no gate, no RoPE)
    hc = layer_norm(x, f(w["ln3_gamma"]), f(w["ln3_beta"]))
    qc = rms_norm(linear(hc, f(w["W_cq"]), f(w["b_cq"])), f(w["g_cq"]))
    L_t = text_k.shape[0]
    cross = attention_dense(qc.reshape(L, H, D), f(text_k).reshape(L_t, H, D),
                            f(text_v).reshape(L_t, H, D)).reshape(L, C)
    upd_cross = linear(cross, f(w["W_co"]), f(w["b_co"]))
    x = x + upd_cross

    # feed-forward branch
    h2 = layer_norm(x) * (1.0 + scale2) + shift2
    u = gelu_tanh(linear(h2, f(w["W_1"]), f(w["b_1"])))
    upd_ffn = gate2 * linear(u, f(w["W_2"]), f(w["b_2"]))
    x = x + upd_ffn

    if debug is not None:
        # what each of the three branches added to x (tests check that none of them hides below the tolerance)
        debug.update(h=h, q=q.reshape(L, C), k=k, v=v, attn=attn, qc=qc, cross=cross, u=u,
                     upd_self=upd_self, upd_cross=upd_cross, upd_ffn=upd_ffn)
    return x


# --------------------------------------------------------------------------- conditioning and the step
def timestep_embedding(t, dim=256, dtype=np.float64):
    """[cos(t w_j) for j < dim/2] ++ [sin(t w_j)],  w_j = 10000**(-j/(dim/2))."""
    half = dim // 2
    j = np.arange(half, dtype=np.float64)
    arg = float(t) * ROPE_BASE ** (-j / half)
    return np.concatenate([np.cos(arg), np.sin(arg)]).astype(dtype)


def timestep_vector(mw, t, dtype=np.float64):
    """tvec = Lin2(SiLU(Lin1(timestep_embedding(t)))), the ``[C]`` vector every modulation is made from."""
    f = lambda a: np.asarray(a, dtype=dtype)
    emb = timestep_embedding(t, f(mw["W_t1"]).shape[1], dtype)
    return linear(silu(linear(emb, f(mw["W_t1"]), f(mw["b_t1"]))), f(mw["W_t2"]), f(mw["b_t2"]))


def conditioning(mw, t=None, tvec=None, dtype=np.float64):
    """Timestep -> tvec -> e0 ``[6, C]``.

    tvec = Lin2(SiLU(Lin1(timestep_embedding(t))));  e0 = Lin_mod(SiLU(tvec)).
    If ``tvec`` is given the first stage is skipped.
    """
    f = lambda a: np.asarray(a, dtype=dtype)
    if tvec is None:
        tvec = timestep_vector(mw, t, dtype)
    tvec = f(tvec)
    C = tvec.shape[-1]
    return linear(silu(tvec), f(mw["W_mod"]), f(mw["b_mod"])).reshape(6, C)


def denoise_step(x, mw, block_ws, caches, text_ks, text_vs, n_heads, tokens_per_frame, grid_w,
                 frame_pos0, advance=True, t=None, tvec=None, dtype=np.float64):
    """Conditioning, then blocks 0..N-1 in sequence, each with its own cache."""
    e0 = conditioning(mw, t=t, tvec=tvec, dtype=dtype)
    for layer, w in enumerate(block_ws):
        x = dit_block_forward(x, e0, w, caches[layer], text_ks[layer], text_vs[layer], n_heads,
                              tokens_per_frame, grid_w, frame_pos0, advance=advance, dtype=dtype)
    return x
