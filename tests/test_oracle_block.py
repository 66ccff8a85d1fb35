"""Pins of the DiT-block oracle (CPU only).

Each oracle function is checked against something that is not itself: PyTorch
library routines for the pieces that have one, closed forms and invariants for
RoPE and the softmax, a scalar brute-force evaluation of a tiny block written
with explicit sums, and the structural statements the paper makes about the
cache (a window that holds all history is full block-causal attention; sink
tokens stay; a repeated denoising step moves nothing).
"""

import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import RollingKVCache
from paper_2511_07399_amd import workloads as wk

T64 = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ pointwise pieces vs library routines
def test_layer_norm_matches_torch():
    x = rng(1).normal(size=(7, 48)) * 3 + 0.7
    g, b = rng(2).normal(size=48), rng(3).normal(size=48)
    np.testing.assert_allclose(oracle.layer_norm(x), F.layer_norm(T64(x), (48,), eps=1e-6).numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.layer_norm(x, g, b),
                               F.layer_norm(T64(x), (48,), T64(g), T64(b), eps=1e-6).numpy(), atol=1e-12)
    y = oracle.layer_norm(x)
    assert abs(y.mean(-1)).max() < 1e-12 and abs(y.var(-1) - 1).max() < 1e-5


def test_rms_norm_matches_torch():
    x = rng(4).normal(size=(5, 64)) * 2
    g = rng(5).normal(size=64)
    np.testing.assert_allclose(oracle.rms_norm(x, g), F.rms_norm(T64(x), (64,), T64(g), eps=1e-6).numpy(), atol=1e-12)


def test_gelu_and_silu_match_torch():
    x = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(oracle.gelu_tanh(x), F.gelu(T64(x), approximate="tanh").numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.silu(x), F.silu(T64(x)).numpy(), atol=1e-12)
    # the tanh form is within 1e-3 of the erf form: the flavour cannot matter at the 2e-2 bar
    assert abs(oracle.gelu_tanh(x) - F.gelu(T64(x)).numpy()).max() < 1e-3


# ------------------------------------------------------------------ RoPE
def test_rope_pair_split():
    assert oracle.rope_pair_split(128) == (22, 21, 21)
    assert sum(oracle.rope_pair_split(12)) == 6


def test_rope_identity_at_origin_and_norm_preserving():
    x = rng(6).normal(size=(9, 3, 128))
    pos0 = np.zeros((9, 3), dtype=np.int64)
    np.testing.assert_array_equal(oracle.rope_3d(x, pos0), x)
    pos = rng(7).integers(0, 500, size=(9, 3))
    y = oracle.rope_3d(x, pos)
    pair_norm = lambda a: a[..., 0::2] ** 2 + a[..., 1::2] ** 2
    np.testing.assert_allclose(pair_norm(y), pair_norm(x), rtol=1e-12)


def test_rope_angles_closed_form():
    """A unit vector (1, 0) in every pair turns to (cos, sin) of pos * 10000^(-j/d_axis)."""
    D = 128
    x = np.zeros((1, 1, D))
    x[..., 0::2] = 1.0
    pf, pr, pc = 37, 5, 11
    y = oracle.rope_3d(x, np.array([[pf, pr, pc]]))[0, 0]
    p = 0
    for pos_a, d_a in ((pf, 22), (pr, 21), (pc, 21)):
        for j in range(d_a):
            ang = pos_a * 10000.0 ** (-j / d_a)
            assert y[2 * p] == pytest.approx(math.cos(ang), abs=1e-12)
            assert y[2 * p + 1] == pytest.approx(math.sin(ang), abs=1e-12)
            p += 1
    assert p == 64
    # (0, 1) turns to (-sin, cos): fixes the sign of the rotation
    x2 = np.zeros((1, 1, D))
    x2[..., 1::2] = 1.0
    y2 = oracle.rope_3d(x2, np.array([[pf, 0, 0]]))[0, 0]
    assert y2[0] == pytest.approx(-math.sin(pf), abs=1e-12) and y2[1] == pytest.approx(math.cos(pf), abs=1e-12)
    assert y2[44] == 0.0 and y2[45] == 1.0        # row/col pairs untouched at row = col = 0


def test_rope_matches_complex_rotation():
    """Interleaved pairs as complex numbers times exp(i theta) (torch.view_as_complex)."""
    L, H, D = 6, 2, 128
    x = rng(8).normal(size=(L, H, D))
    pos = rng(9).integers(0, 90, size=(L, 3))
    theta = torch.cat([T64(pos[:, a:a + 1]) * (10000.0 ** (-torch.arange(d, dtype=torch.float64) / d))[None]
                       for a, d in enumerate((22, 21, 21))], dim=1)
    rot = torch.polar(torch.ones_like(theta), theta)[:, None, :]
    want = torch.view_as_real(torch.view_as_complex(T64(x).reshape(L, H, D // 2, 2)) * rot).reshape(L, H, D)
    np.testing.assert_allclose(oracle.rope_3d(x, pos), want.numpy(), atol=1e-12)


def test_rope_scores_depend_on_position_differences_only():
    L, H, D = 5, 2, 128
    q, k = rng(10).normal(size=(L, H, D)), rng(11).normal(size=(L, H, D))
    pq, pk = rng(12).integers(0, 40, size=(L, 3)), rng(13).integers(0, 40, size=(L, 3))
    shift = np.array([[123, 7, 9]])
    s0 = np.einsum("qhd,khd->hqk", oracle.rope_3d(q, pq), oracle.rope_3d(k, pk))
    s1 = np.einsum("qhd,khd->hqk", oracle.rope_3d(q, pq + shift), oracle.rope_3d(k, pk + shift))
    np.testing.assert_allclose(s0, s1, atol=1e-9)


def test_token_positions():
    from oracle.dit_block import token_positions
    pos = token_positions(12, 6, 3, frame_pos0=10)          # 2 frames of 2x3 tokens
    assert pos[0].tolist() == [10, 0, 0] and pos[2].tolist() == [10, 0, 2]
    assert pos[3].tolist() == [10, 1, 0] and pos[5].tolist() == [10, 1, 2]
    assert pos[6].tolist() == [11, 0, 0] and pos[11].tolist() == [11, 1, 2]


# ------------------------------------------------------------------ attention
def test_attention_matches_torch_sdpa_and_rows_sum_to_one():
    Lq, Lk, H, D = 7, 19, 3, 16
    q, k, v = (rng(s).normal(size=(n, H, D)) for s, n in ((14, Lq), (15, Lk), (16, Lk)))
    out, probs = oracle.attention_dense(q, k, v, return_probs=True)
    want = F.scaled_dot_product_attention(T64(q).transpose(0, 1), T64(k).transpose(0, 1), T64(v).transpose(0, 1))
    np.testing.assert_allclose(out, want.transpose(0, 1).numpy(), atol=1e-12)
    np.testing.assert_allclose(probs.sum(-1), 1.0, atol=1e-14)
    assert probs.min() >= 0
    # the order in which keys are listed does not matter (the GPU scans physical slot order)
    perm = rng(17).permutation(Lk)
    np.testing.assert_allclose(oracle.attention_dense(q, k[perm], v[perm]), out, atol=1e-12)


# ------------------------------------------------------------------ tiny block, scalar brute force
TINY = wk.Workload("brute", C=24, H=2, F=16, grid_h=1, grid_w=2, frames_per_chunk=2, sink_frames=1,
                   window_frames=3, L_t=3, B=1, N=1, steps=(1,), chunks=3, t_dim=8)


def tiny_setup(wl, seed=0, scale=8.0):
    """Weights as float64 numpy; scaled up so that every term matters in a tiny model."""
    w = wk.to_numpy(wk.block_weights(wl, 0, seed))
    for name in w:
        if name.startswith(("W_", "b_", "mod", "ln3_beta")):
            w[name] = w[name] * scale
    return w


def brute_block(x, e0, w, resident_k, resident_v, text_k, text_v, H, P, grid_w, frame_pos0):
    """Scalar evaluation of one block.  resident_k/v: lists of earlier rows (already final)."""
    L, C = len(x), len(x[0])
    D = C // H
    dot = lambda a, b: sum(p * q for p, q in zip(a, b))
    lin = lambda vec, W, b: [dot(vec, W[o]) + b[o] for o in range(len(W))]

    def ln(vec):
        m = sum(vec) / len(vec)
        var = sum((t - m) ** 2 for t in vec) / len(vec)
        return [(t - m) / math.sqrt(var + 1e-6) for t in vec]

    def rms(vec, g):
        r = math.sqrt(sum(t * t for t in vec) / len(vec) + 1e-6)
        return [t / r * gg for t, gg in zip(vec, g)]

    def rope(vec, i):
        f, r, c = frame_pos0 + i // P, (i % P) // grid_w, (i % P) % grid_w
        pairs = D // 2
        third = pairs // 3
        counts = (pairs - 2 * third, third, third)
        out = list(vec)
        for h in range(H):
            p = 0
            for position, d_a in zip((f, r, c), counts):
                for j in range(d_a):
                    ang = position * 10000.0 ** (-j / d_a)
                    a, b = vec[h * D + 2 * p], vec[h * D + 2 * p + 1]
                    out[h * D + 2 * p] = a * math.cos(ang) - b * math.sin(ang)
                    out[h * D + 2 * p + 1] = a * math.sin(ang) + b * math.cos(ang)
                    p += 1
        return out

    def attend(qrow, keys, vals):
        out = [0.0] * C
        for h in range(H):
            sl = slice(h * D, (h + 1) * D)
            s = [dot(qrow[sl], kr[sl]) / math.sqrt(D) for kr in keys]
            mx = max(s)
            e = [math.exp(t - mx) for t in s]
            z = sum(e)
            for d in range(D):
                out[h * D + d] = sum(e[n] / z * vals[n][h * D + d] for n in range(len(keys)))
        return out

    mod = [[w["mod_table"][r][c] + e0[r][c] for c in range(C)] for r in range(6)]
    gelu = lambda t: 0.5 * t * (1 + math.tanh(math.sqrt(2 / math.pi) * (t + 0.044715 * t ** 3)))
    qs, new_k, new_v = [], [], []
    for i in range(L):
        h = [n * (1 + mod[1][c]) + mod[0][c] for c, n in enumerate(ln(x[i]))]
        qs.append(rope(rms(lin(h, w["W_q"], w["b_q"]), w["g_q"]), i))
        new_k.append(rope(rms(lin(h, w["W_k"], w["b_k"]), w["g_k"]), i))
        new_v.append(lin(h, w["W_v"], w["b_v"]))
    keys, vals = resident_k + new_k, resident_v + new_v
    out = []
    for i in range(L):
        a = attend(qs[i], keys, vals)
        y = [x[i][c] + mod[2][c] * t for c, t in enumerate(lin(a, w["W_o"], w["b_o"]))]
        hc = [n * w["ln3_gamma"][c] + w["ln3_beta"][c] for c, n in enumerate(ln(y))]
        qc = rms(lin(hc, w["W_cq"], w["b_cq"]), w["g_cq"])
        cr = attend(qc, text_k, text_v)
        y = [y[c] + t for c, t in enumerate(lin(cr, w["W_co"], w["b_co"]))]
        h2 = [n * (1 + mod[4][c]) + mod[3][c] for c, n in enumerate(ln(y))]
        u = [gelu(t) for t in lin(h2, w["W_1"], w["b_1"])]
        y = [y[c] + mod[5][c] * t for c, t in enumerate(lin(u, w["W_2"], w["b_2"]))]
        out.append(y)
    return out, new_k, new_v


def test_block_matches_scalar_brute_force_over_a_stream_with_eviction():
    wl = TINY
    w = tiny_setup(wl)
    wl_lists = {k: v.tolist() for k, v in w.items()}
    ctx = wk.text_context(wl).double().numpy()
    # text K/V by brute force as well
    dot = lambda a, b: sum(p * q for p, q in zip(a, b))
    tk, tv = [], []
    for row in ctx.tolist():
        kk = [dot(row, w["W_ck"][o].tolist()) + w["b_ck"][o] for o in range(wl.C)]
        r = math.sqrt(sum(t * t for t in kk) / wl.C + 1e-6)
        tk.append([t / r * g for t, g in zip(kk, w["g_ck"])])
        tv.append([dot(row, w["W_cv"][o].tolist()) + w["b_cv"][o] for o in range(wl.C)])
    text_k, text_v = oracle.text_kv_prepare(ctx, w)
    np.testing.assert_allclose(text_k, np.array(tk), atol=1e-12)
    np.testing.assert_allclose(text_v, np.array(tv), atol=1e-12)

    cache = RollingKVCache(wl.S, wl.W, wl.P, wl.C)
    hist_k, hist_v = [], []            # every final k/v row ever produced, by token id
    for chunk in range(4):             # 2 + 4*... tokens: S=2, W=6, L=4 -> eviction from chunk 2 on
        x = wk.chunk_input(wl, chunk).double().numpy()
        e0 = (wk._normal((6, wl.C), 77 + chunk).double().numpy()) * 0.5
        got = oracle.dit_block_forward(x, e0, w, cache, text_k, text_v, wl.H, wl.P, wl.grid_w,
                                       frame_pos0=chunk * wl.frames_per_chunk)
        total_before = chunk * wl.L
        # resident set by definition: sink ids + the last (W - L) ids before this chunk
        ids = [g for g in range(total_before) if g < wl.S or g >= max(wl.S, total_before + wl.L - wl.W)]
        want, nk, nv = brute_block(x.tolist(), e0.tolist(), wl_lists, [hist_k[g] for g in ids],
                                   [hist_v[g] for g in ids], tk, tv, wl.H, wl.P, wl.grid_w,
                                   chunk * wl.frames_per_chunk)
        hist_k += nk
        hist_v += nv
        np.testing.assert_allclose(got, np.array(want), rtol=1e-10, atol=1e-10)
        assert abs(got - x).max() > 0.1          # the branches really contribute in this setting
    assert cache.state()["evicted"] == 4 * wl.L - wl.S - wl.W > 0


# ------------------------------------------------------------------ structural statements about the cache
def stream_block(wl, w, n_chunks, S, W, seed=0, advance_pattern=None):
    ctx = wk.text_context(wl, base_seed=seed).double().numpy()
    text_k, text_v = oracle.text_kv_prepare(ctx, w)
    cache = RollingKVCache(S, W, wl.P, wl.C)
    outs, dbg = [], []
    for chunk in range(n_chunks):
        x = wk.chunk_input(wl, chunk, base_seed=seed).double().numpy()
        e0 = wk._normal((6, wl.C), 900 + chunk).double().numpy() * 0.3
        d = {}
        outs.append(oracle.dit_block_forward(x, e0, w, cache, text_k, text_v, wl.H, wl.P, wl.grid_w,
                                             frame_pos0=chunk * wl.frames_per_chunk, debug=d))
        dbg.append(d)
    return outs, dbg, cache


MID = wk.Workload("mid", C=64, H=2, F=96, grid_h=2, grid_w=3, frames_per_chunk=1, sink_frames=1,
                  window_frames=2, L_t=5, B=1, N=1, steps=(1,), chunks=5)


def test_window_holding_all_history_is_full_block_causal_attention():
    wl = MID
    w = tiny_setup(wl, scale=4.0)
    n = 5
    _, dbg, cache = stream_block(wl, w, n, S=wl.P, W=n * wl.P)
    assert cache.state()["evicted"] == 0
    H, D, L = wl.H, wl.D, wl.L
    q = torch.cat([T64(d["q"]) for d in dbg]).reshape(n * L, H, D).transpose(0, 1)
    k = torch.cat([T64(d["k"]) for d in dbg]).reshape(n * L, H, D).transpose(0, 1)
    v = torch.cat([T64(d["v"]) for d in dbg]).reshape(n * L, H, D).transpose(0, 1)
    blk = torch.arange(n * L) // L
    mask = blk[:, None] >= blk[None, :]                     # block lower triangular
    want = F.scaled_dot_product_attention(q, k, v, attn_mask=mask).transpose(0, 1).reshape(n * L, wl.C)
    got = np.concatenate([d["attn"] for d in dbg])
    np.testing.assert_allclose(got, want.numpy(), atol=1e-11)


def test_no_sink_and_window_of_one_chunk_is_plain_self_attention():
    wl = MID
    w = tiny_setup(wl, scale=4.0)
    _, dbg, _ = stream_block(wl, w, 3, S=0, W=wl.L)
    for d in dbg:
        q, k, v = (T64(d[n]).reshape(wl.L, wl.H, wl.D).transpose(0, 1) for n in ("q", "k", "v"))
        want = F.scaled_dot_product_attention(q, k, v).transpose(0, 1).reshape(wl.L, wl.C)
        np.testing.assert_allclose(d["attn"], want.numpy(), atol=1e-11)


def test_rolling_window_attends_to_sink_plus_recent_frames_only():
    """With eviction, chunk t sees frame 0 (sink) and frames t-1, t: checked with a masked library call."""
    wl = MID
    w = tiny_setup(wl, scale=4.0)
    n = 5
    _, dbg, cache = stream_block(wl, w, n, S=wl.P, W=2 * wl.P)
    assert cache.state()["evicted"] == (n - 3) * wl.P
    H, D, L = wl.H, wl.D, wl.L
    cat = lambda name: torch.cat([T64(d[name]) for d in dbg]).reshape(n * L, H, D).transpose(0, 1)
    blk = torch.arange(n * L) // L
    qb, kb = blk[:, None], blk[None, :]
    mask = (kb == 0) & (qb >= 0) | ((kb <= qb) & (kb >= qb - 1))
    want = F.scaled_dot_product_attention(cat("q"), cat("k"), cat("v"), attn_mask=mask)
    got = np.concatenate([d["attn"] for d in dbg])
    np.testing.assert_allclose(got, want.transpose(0, 1).reshape(n * L, wl.C).numpy(), atol=1e-11)


def test_zero_gates_leave_x_unchanged_but_cache_is_written():
    wl = MID
    w = tiny_setup(wl, scale=4.0)
    w["W_co"] = w["W_co"] * 0
    w["b_co"] = w["b_co"] * 0
    e0 = -w["mod_table"].copy()
    e0[[0, 1, 3, 4]] += rng(20).normal(size=(4, wl.C))       # shifts and scales arbitrary, gates cancel to 0
    cache = RollingKVCache(wl.S, wl.W, wl.P, wl.C)
    text_k, text_v = oracle.text_kv_prepare(wk.text_context(wl).double().numpy(), w)
    x = wk.chunk_input(wl, 0).double().numpy()
    y = oracle.dit_block_forward(x, e0, w, cache, text_k, text_v, wl.H, wl.P, wl.grid_w, 0)
    np.testing.assert_array_equal(y, x)
    assert cache.state()["total"] == wl.L and not np.isnan(cache.gather()[0]).any()


def test_block_matches_composition_of_torch_library_ops():
    """The whole block rebuilt from torch.nn.functional pieces and complex-number RoPE."""
    wl = MID
    w = tiny_setup(wl, scale=4.0)
    tw = {k: T64(v) for k, v in w.items()}
    text_k, text_v = oracle.text_kv_prepare(wk.text_context(wl).double().numpy(), w)
    cache = RollingKVCache(wl.S, 4 * wl.P, wl.P, wl.C)       # no eviction in this test
    H, D, C, L = wl.H, wl.D, wl.C, wl.L
    past_k, past_v = [], []
    for chunk in range(3):
        x = wk.chunk_input(wl, chunk).double().numpy()
        e0 = wk._normal((6, C), 50 + chunk).double().numpy() * 0.4
        got = oracle.dit_block_forward(x, e0, w, cache, text_k, text_v, H, wl.P, wl.grid_w, frame_pos0=7 + chunk)
        m = tw["mod_table"] + T64(e0)
        xt = T64(x)
        h = F.layer_norm(xt, (C,), eps=1e-6) * (1 + m[1]) + m[0]
        i = torch.arange(L)
        pos = torch.stack([7 + chunk + i // wl.P, (i % wl.P) // wl.grid_w, (i % wl.P) % wl.grid_w], 1).double()
        dsplit = oracle.rope_pair_split(D)
        theta = torch.cat([pos[:, a:a + 1] * (10000.0 ** (-torch.arange(d, dtype=torch.float64) / d))[None]
                           for a, d in enumerate(dsplit)], 1)
        rot = torch.polar(torch.ones_like(theta), theta)[:, None, :]
        rope = lambda t: torch.view_as_real(torch.view_as_complex(t.reshape(L, H, D // 2, 2)) * rot).reshape(L, C)
        q = rope(F.rms_norm(F.linear(h, tw["W_q"], tw["b_q"]), (C,), tw["g_q"], eps=1e-6))
        k = rope(F.rms_norm(F.linear(h, tw["W_k"], tw["b_k"]), (C,), tw["g_k"], eps=1e-6))
        v = F.linear(h, tw["W_v"], tw["b_v"])
        past_k.append(k)
        past_v.append(v)
        heads = lambda t: t.reshape(-1, H, D).transpose(0, 1)
        a = F.scaled_dot_product_attention(heads(q), heads(torch.cat(past_k)), heads(torch.cat(past_v)))
        xt = xt + m[2] * F.linear(a.transpose(0, 1).reshape(L, C), tw["W_o"], tw["b_o"])
        hc = F.layer_norm(xt, (C,), tw["ln3_gamma"], tw["ln3_beta"], eps=1e-6)
        qc = F.rms_norm(F.linear(hc, tw["W_cq"], tw["b_cq"]), (C,), tw["g_cq"], eps=1e-6)
        cr = F.scaled_dot_product_attention(heads(qc), heads(T64(text_k)), heads(T64(text_v)))
        xt = xt + F.linear(cr.transpose(0, 1).reshape(L, C), tw["W_co"], tw["b_co"])
        h2 = F.layer_norm(xt, (C,), eps=1e-6) * (1 + m[4]) + m[3]
        xt = xt + m[5] * F.linear(F.gelu(F.linear(h2, tw["W_1"], tw["b_1"]), approximate="tanh"), tw["W_2"], tw["b_2"])
        np.testing.assert_allclose(got, xt.numpy(), atol=1e-10)


def test_repeated_denoising_step_moves_nothing_and_keeps_last_values():
    wl = MID
    w = tiny_setup(wl, scale=4.0)
    text_k, text_v = oracle.text_kv_prepare(wk.text_context(wl).double().numpy(), w)
    cache = RollingKVCache(wl.S, wl.W, wl.P, wl.C)
    e0 = wk._normal((6, wl.C), 5).double().numpy() * 0.3
    for chunk in range(4):
        x = wk.chunk_input(wl, chunk).double().numpy()
        x1 = oracle.dit_block_forward(x, e0, w, cache, text_k, text_v, wl.H, wl.P, wl.grid_w, chunk, advance=True)
        st, sm = cache.state(), cache.slot_map().copy()
        d = {}
        oracle.dit_block_forward(x1, e0, w, cache, text_k, text_v, wl.H, wl.P, wl.grid_w, chunk,
                                 advance=False, debug=d)
        assert cache.state() == st
        np.testing.assert_array_equal(cache.slot_map(), sm)
        k_res, v_res = cache.gather()
        np.testing.assert_array_equal(k_res[-wl.L:], d["k"])      # the last step's values persist
        np.testing.assert_array_equal(v_res[-wl.L:], d["v"])
    assert cache.state()["total"] == 4 * wl.L


# ------------------------------------------------------------------ conditioning and the step
def test_timestep_embedding_closed_form():
    e = oracle.timestep_embedding(0.0)
    np.testing.assert_array_equal(e[:128], 1.0)
    np.testing.assert_array_equal(e[128:], 0.0)
    t = 613.25
    e = oracle.timestep_embedding(t)
    assert e[0] == pytest.approx(math.cos(t), abs=1e-12) and e[128] == pytest.approx(math.sin(t), abs=1e-12)
    w127 = 10000.0 ** (-127 / 128)
    assert e[127] == pytest.approx(math.cos(t * w127), abs=1e-12)
    assert e[255] == pytest.approx(math.sin(t * w127), abs=1e-12)
    assert e[64] == pytest.approx(math.cos(t * 0.01), abs=1e-12)


def test_conditioning_matches_torch_composition():
    wl = MID
    mw = wk.to_numpy(wk.model_weights(wl))
    for k in mw:
        mw[k] = mw[k] * 6.0
    t = 321.5
    tm = {k: T64(v) for k, v in mw.items()}
    emb = T64(oracle.timestep_embedding(t, wl.t_dim))
    tvec = F.linear(F.silu(F.linear(emb, tm["W_t1"], tm["b_t1"])), tm["W_t2"], tm["b_t2"])
    want = F.linear(F.silu(tvec), tm["W_mod"], tm["b_mod"]).reshape(6, wl.C)
    np.testing.assert_allclose(oracle.conditioning(mw, t=t), want.numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.conditioning(mw, tvec=tvec.numpy()), want.numpy(), atol=1e-12)
    # row r of e0 is outputs [r*C, (r+1)*C) of the modulation projection
    assert oracle.conditioning(mw, t=t)[2, 5] == pytest.approx(float(F.linear(F.silu(tvec), tm["W_mod"], tm["b_mod"])[2 * wl.C + 5]))


def test_denoise_step_is_conditioning_then_blocks_in_order():
    wl = wk.Workload("mid3", C=64, H=2, F=96, grid_h=2, grid_w=3, frames_per_chunk=1, sink_frames=1,
                     window_frames=2, L_t=5, B=1, N=3, steps=(1,), chunks=2)
    mw = wk.to_numpy(wk.model_weights(wl))
    bws = [tiny_setup(wl, seed=0, scale=4.0) for _ in range(wl.N)]
    for layer in range(wl.N):
        bws[layer] = {k: v * 1.0 for k, v in wk.to_numpy(wk.block_weights(wl, layer)).items()}
    ctx = wk.text_context(wl).double().numpy()
    tks, tvs = zip(*(oracle.text_kv_prepare(ctx, w) for w in bws))
    caches = [RollingKVCache(wl.S, wl.W, wl.P, wl.C) for _ in range(wl.N)]
    caches2 = [RollingKVCache(wl.S, wl.W, wl.P, wl.C) for _ in range(wl.N)]
    x = wk.chunk_input(wl, 0).double().numpy()
    got = oracle.denoise_step(x, mw, bws, caches, tks, tvs, wl.H, wl.P, wl.grid_w, 0, t=500.0)
    e0 = oracle.conditioning(mw, t=500.0)
    y = x
    for layer in range(wl.N):
        y = oracle.dit_block_forward(y, e0, bws[layer], caches2[layer], tks[layer], tvs[layer], wl.H, wl.P,
                                     wl.grid_w, 0)
    np.testing.assert_array_equal(got, y)
    assert all(c.state()["total"] == wl.L for c in caches)


def test_float32_run_of_the_oracle_agrees_with_float64():
    """The oracle's own rounding in fp32 is far below the 2e-2 parity bar."""
    wl = wk.WORKLOADS["tiny"]
    w = wk.to_numpy(wk.block_weights(wl, 0))
    ctx = wk.text_context(wl).double().numpy()
    outs = {}
    for dt in (np.float64, np.float32):
        text_k, text_v = oracle.text_kv_prepare(ctx, w, dtype=dt)
        cache = RollingKVCache(wl.S, wl.W, wl.P, wl.C, dtype=dt)
        mw = wk.to_numpy(wk.model_weights(wl))
        ys = []
        for chunk in range(4):
            e0 = oracle.conditioning(mw, tvec=wk.timestep_vector(wl, chunk).double().numpy(), dtype=dt)
            x = wk.chunk_input(wl, chunk).double().numpy()
            ys.append(oracle.dit_block_forward(x, e0, w, cache, text_k, text_v, wl.H, wl.P, wl.grid_w, chunk, dtype=dt))
        outs[dt] = np.stack(ys)
        assert outs[dt].dtype == dt
    err = abs(outs[np.float32] - outs[np.float64]).max() / abs(outs[np.float64]).max()
    assert err < 1e-5
