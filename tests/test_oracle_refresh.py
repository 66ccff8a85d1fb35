"""Pins of the sink-refresh / RoPE-refresh oracle (CPU only).

The paper prints no numbers for these mechanisms, so the pins are closed forms (cosines of constructed vectors,
the threshold rule case by case, the index rule of the RoPE reset), brute force with explicit sums, and the one
invariance that fixes the direction of the key rotation: attention depends on rotary phase *differences* only, so a
block evaluated at frame f on a cache equals the block evaluated at frame f - delta on the cache moved by delta.
"""

import copy
import math

import numpy as np
import pytest

import oracle
from oracle import RollingKVCache
from oracle import refresh
from paper_2511_07399_amd import workloads as wk


def rng(seed):
    return np.random.default_rng(seed)


def filled_cache(P=4, C=8, sink_frames=2, window_frames=3, frames=(2, 1, 1), seed=0):
    """A cache after a few appends of ``frames[i]`` frames each; returns (cache, list of (k, v) per append)."""
    c = RollingKVCache(sink_frames * P, window_frames * P, P, C)
    g = rng(seed)
    hist = []
    for f in frames:
        k, v = g.normal(size=(f * P, C)), g.normal(size=(f * P, C))
        c.append_evict(k, v)
        hist.append((k, v))
    return c, hist


# ------------------------------------------------------------------ cosine
def test_cosine_closed_forms_and_brute_force():
    a = rng(1).normal(size=37)
    assert refresh.cosine(a, a) == pytest.approx(1.0, abs=1e-15)
    assert refresh.cosine(a, -a) == pytest.approx(-1.0, abs=1e-15)
    assert refresh.cosine(a, 3.5 * a) == pytest.approx(1.0, abs=1e-15)          # scale free
    e0, e1 = np.eye(5)[0], np.eye(5)[1]
    assert refresh.cosine(e0, e1) == 0.0
    assert refresh.cosine(e0 + e1, e0) == pytest.approx(1 / math.sqrt(2), abs=1e-15)   # 45 degrees
    assert refresh.cosine(np.zeros(5), e0) == 0.0
    b = rng(2).normal(size=37)
    dot = sum(float(x) * float(y) for x, y in zip(a, b))
    na = math.sqrt(sum(float(x) ** 2 for x in a))
    nb = math.sqrt(sum(float(y) ** 2 for y in b))
    assert refresh.cosine(a, b) == pytest.approx(dot / (na * nb), abs=1e-14)


def test_similarity_is_taken_over_value_rows_of_whole_frames():
    P, C = 4, 8
    c = RollingKVCache(2 * P, 3 * P, P, C)
    g = rng(3)
    k0, v0 = g.normal(size=(2 * P, C)), g.normal(size=(2 * P, C))
    c.append_evict(k0, v0)                                     # two frames: both go to the sink
    # a new frame whose values equal sink frame 1's, with unrelated keys
    c.append_evict(g.normal(size=(P, C)) * 50, v0[P:].copy())
    alpha = oracle.sink_similarity(c)
    assert alpha.shape == (2,)
    assert alpha[1] == pytest.approx(1.0, abs=1e-14)
    want0 = refresh.cosine(v0[P:].reshape(-1), v0[:P].reshape(-1))
    assert alpha[0] == pytest.approx(want0, abs=1e-14) and abs(alpha[0]) < 0.9
    # token order inside the frame matters (it is one flattened vector, not a bag of tokens)
    c.append_evict(g.normal(size=(P, C)), v0[P:][::-1].copy())
    assert oracle.sink_similarity(c)[1] < 0.9


def test_frame_back_counts_from_the_end_of_the_latest_append():
    P, C = 3, 4
    c = RollingKVCache(P, 6 * P, P, C)
    g = rng(4)
    c.append_evict(g.normal(size=(P, C)), g.normal(size=(P, C)))           # the sink frame
    k, v = g.normal(size=(3 * P, C)), g.normal(size=(3 * P, C))
    c.append_evict(k, v)
    for back, first_row in ((0, 2 * P), (1, P), (2, 0)):
        ids, rows = c.frame_rows(back)
        assert ids == list(range(P + first_row, P + first_row + P))
        np.testing.assert_array_equal(np.stack([r[1] for r in rows]), v[first_row:first_row + P])
    with pytest.raises(ValueError):
        c.frame_rows(3)
    # a frame that was stored in the sink itself cannot serve as h_t
    c2 = RollingKVCache(P, 2 * P, P, C)
    c2.append_evict(g.normal(size=(P, C)), g.normal(size=(P, C)))
    with pytest.raises(RuntimeError):
        c2.frame_rows(0)


# ------------------------------------------------------------------ the update rule
def test_threshold_rule_keeps_at_or_above_tau_and_replaces_below():
    c, hist = filled_cache()
    alpha = oracle.sink_similarity(c)
    lo, hi = sorted(alpha)
    before = c.slot_contents()
    state = c.state()
    # tau equal to the smaller alpha: alpha_i >= tau for both, nothing changes
    a, replaced = oracle.adaptive_sink_update(copy.deepcopy(c), tau=lo)
    assert replaced == []
    # tau between the two: exactly the less similar sink is replaced
    c1 = copy.deepcopy(c)
    a, replaced = oracle.adaptive_sink_update(c1, tau=(lo + hi) / 2)
    worst = int(np.argmin(alpha))
    assert replaced == [worst]
    np.testing.assert_array_equal(a, alpha)
    P = c.P
    k1, v1 = c1.slot_contents()
    src_k, src_v = hist[-1]
    np.testing.assert_array_equal(k1[worst * P:(worst + 1) * P], src_k)        # s_i = h_t: keys and values
    np.testing.assert_array_equal(v1[worst * P:(worst + 1) * P], src_v)
    other = 1 - worst
    np.testing.assert_array_equal(k1[other * P:(other + 1) * P], before[0][other * P:(other + 1) * P])
    np.testing.assert_array_equal(k1[c.S:], before[0][c.S:])                   # the window is untouched
    assert c1.state() == state                                                   # counters do not move
    sm = c1.slot_map()
    np.testing.assert_array_equal(sm[worst * P:(worst + 1) * P], np.arange(c.total - P, c.total))
    # tau above both: every sink becomes h_t
    c2 = copy.deepcopy(c)
    _, replaced = oracle.adaptive_sink_update(c2, tau=1.1)
    assert replaced == [0, 1]
    # NaN similarity never counts as "similar enough"
    assert not (float("nan") >= 0.5)


def test_refreshed_sink_is_attended_and_survives_eviction_of_its_source():
    c, hist = filled_cache()
    P, C = c.P, c.width
    oracle.refresh_sink(c, 0)
    src_k, src_v = hist[-1]
    k, v = c.gather()
    assert k.shape[0] == c.S + len(c.window_ids)
    np.testing.assert_array_equal(k[:P], src_k)                 # sink frame 0, first in the resident order
    np.testing.assert_array_equal(k[-P:], src_k)                # and still the newest window frame: resident twice
    g = rng(9)
    for _ in range(5):                                          # push the source frame out of the window
        c.append_evict(g.normal(size=(P, C)), g.normal(size=(P, C)))
    assert c.state()["evicted"] > 0
    k, v = c.gather()
    np.testing.assert_array_equal(k[:P], src_k)
    np.testing.assert_array_equal(v[:P], src_v)
    assert not any(np.array_equal(k[i:i + P], src_k) for i in range(P, k.shape[0] - P + 1, P))


def test_counters_ignore_the_sink_copy_of_a_window_token():
    """The frame copied into the sink is still the oldest window frame: its id is in the slot map twice, and the
    window's oldest slot is the one in the ring part."""
    P, C = 4, 8
    c = RollingKVCache(P, 2 * P, P, C)
    g = rng(11)
    for _ in range(3):
        c.append_evict(g.normal(size=(P, C)), g.normal(size=(P, C)))
    before = c.state()
    c.append_evict(g.normal(size=(2 * P, C)), g.normal(size=(2 * P, C)))       # two frames: the window, wrapped
    st = c.state()
    oracle.refresh_sink(c, 0, frame_back=1)                                     # frame_back 1 = the oldest window frame
    assert c.state() == st and st["oldest_slot"] >= c.S
    sm = c.slot_map()
    assert list(sm[:P]) == list(sm[st["oldest_slot"]:st["oldest_slot"] + P])
    assert before["evicted"] == 0 and st["evicted"] == 2 * P


def test_refresh_closes_the_chunk():
    c, hist = filled_cache()
    k, v = hist[-1]
    c.append_evict(k, v, advance=False)                         # a second denoising step is fine before the refresh
    oracle.refresh_sink(c, 1)
    with pytest.raises(RuntimeError):
        c.append_evict(k, v, advance=False)
    c.append_evict(k, v)                                        # the next chunk opens normally
    c.append_evict(k, v, advance=False)


# ------------------------------------------------------------------ RoPE refresh
def test_rope_refresh_frame_index_rule():
    T = 10
    assert [oracle.rope_refresh_frame(t, T) for t in (0, 9, 10, 11, 15, 20)] == [0, 9, 10, 1, 5, 10]


def test_rotate_keys_is_rope_at_the_shifted_frame_and_touches_frame_pairs_only():
    H, D, P = 2, 128, 3
    C = H * D
    g = rng(5)
    raw = g.normal(size=(2 * P, C))
    pos = oracle.dit_block.token_positions(2 * P, P, 3, frame_pos0=7)          # frames 7 and 8, a 1 x 3 grid
    k = oracle.rope_3d(raw.reshape(-1, H, D), pos).reshape(-1, C)
    v = g.normal(size=(2 * P, C))
    c = RollingKVCache(P, 2 * P, P, C)
    c.append_evict(k, v)
    c0 = copy.deepcopy(c)
    oracle.rotate_keys(c, 5, H)
    k5, v5 = c.slot_contents()
    pos_shift = pos.copy()
    pos_shift[:, 0] -= 5
    want = oracle.rope_3d(raw.reshape(-1, H, D), pos_shift).reshape(-1, C)     # as if cached at frames 2 and 3
    np.testing.assert_allclose(k5[:2 * P], want, atol=1e-12)
    np.testing.assert_array_equal(v5[:2 * P], v)                               # values carry no phase
    # row and column pairs (elements 44 .. 127 of each head) are untouched, frame pairs (0 .. 43) are not
    kk0 = c0.slot_contents()[0][:2 * P].reshape(-1, H, D)
    kk5 = k5[:2 * P].reshape(-1, H, D)
    np.testing.assert_array_equal(kk5[:, :, 44:], kk0[:, :, 44:])
    assert np.abs(kk5[:, :, :44] - kk0[:, :, :44]).max() > 1e-3
    # there and back
    oracle.rotate_keys(c, -5, H)
    np.testing.assert_allclose(c.slot_contents()[0][:2 * P], k, atol=1e-12)


def test_block_output_is_unchanged_by_a_joint_shift_of_cache_and_frame_index():
    """RoPE reset (theta_t -> theta_{t - T_reset}) with the cached keys moved by the same T_reset."""
    wl = wk.Workload("refresh", C=256, H=2, F=384, grid_h=2, grid_w=3, frames_per_chunk=1, sink_frames=1,
                     window_frames=3, L_t=5, B=1, N=1, steps=(1,), chunks=6)
    w = wk.to_numpy(wk.block_weights(wl, 0, 0))
    mw = wk.to_numpy(wk.model_weights(wl, 0))
    ctx = wk.text_context(wl, 0, 0).double().numpy()
    tk, tv = oracle.text_kv_prepare(ctx, w)
    cache = RollingKVCache(wl.S, wl.W, wl.P, wl.C)
    e0 = oracle.conditioning(mw, t=wk.timestep(wl, 0, 0, 0, 0))
    for chunk in range(5):                                                      # frames 0 .. 4, evicting
        x = wk.chunk_input(wl, chunk, 0, 0).double().numpy()
        oracle.dit_block_forward(x, e0, w, cache, tk, tv, wl.H, wl.P, wl.grid_w, chunk)
    x = wk.chunk_input(wl, 5, 0, 0).double().numpy()
    a = copy.deepcopy(cache)
    b = copy.deepcopy(cache)
    ya = oracle.dit_block_forward(x, e0, w, a, tk, tv, wl.H, wl.P, wl.grid_w, 5)
    t_reset = 3
    oracle.rotate_keys(b, t_reset, wl.H)
    yb = oracle.dit_block_forward(x, e0, w, b, tk, tv, wl.H, wl.P, wl.grid_w, oracle.rope_refresh_frame(5, t_reset))
    np.testing.assert_allclose(yb, ya, atol=1e-10)
    # moving the cache the wrong way, or not at all, does change the result
    c = copy.deepcopy(cache)
    oracle.rotate_keys(c, -t_reset, wl.H)
    yc = oracle.dit_block_forward(x, e0, w, c, tk, tv, wl.H, wl.P, wl.grid_w, 5 - t_reset)
    yd = oracle.dit_block_forward(x, e0, w, copy.deepcopy(cache), tk, tv, wl.H, wl.P, wl.grid_w, 5 - t_reset)
    assert np.abs(yc - ya).max() > 1e-6 and np.abs(yd - ya).max() > 1e-6
