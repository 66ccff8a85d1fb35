"""Pins of the rolling-KV-cache oracle (CPU only).

The oracle is a naive list + deque + cursor simulator.  It is pinned here
against what the paper's description fixes (sink tokens persist, the window
rolls first-in-first-out, frame-by-frame; abstract, Section 1, Appendix D) and
against the closed form that follows from it, stated independently below.
"""

import itertools

import numpy as np
import pytest

from oracle import RollingKVCache


# ---- the closed form (a theorem about the cache, not taken from the oracle) ----
def closed_slot(g, S, W):
    return g if g < S else S + (g - S) % W


def closed_state(total, S, W):
    sink_fill = min(total, S)
    win_fill = min(max(total - S, 0), W)
    st = {
        "total": total,
        "sink_fill": sink_fill,
        "win_fill": win_fill,
        "evicted": max(total - S - W, 0),
        "oldest_slot": S + (total - win_fill - S) % W if win_fill else -1,
        "next_slot": closed_slot(total, S, W),
    }
    return st


def closed_slot_map(total, S, W):
    m = np.full(S + W, -1, dtype=np.int64)
    for g in range(total):
        if g < S or g >= max(S, total - W):
            m[closed_slot(g, S, W)] = g
    return m


def rows(ids, width=3):
    """Distinct, recognisable k/v rows for token ids."""
    ids = np.asarray(ids, dtype=np.float64)
    k = ids[:, None] * 10.0 + np.arange(width)[None, :]
    return k, -k


def stream_chunks(cache, sizes):
    g = 0
    for n in sizes:
        k, v = rows(range(g, g + n), cache.width)
        cache.append_evict(k, v, advance=True)
        g += n
        yield g


SMALL = [
    (P, S, W)
    for P in (1, 2, 3)
    for S in (0, P, 2 * P)
    for W in (P, 2 * P, 3 * P, 5 * P)
]


@pytest.mark.parametrize("P,S,W", SMALL)
def test_closed_form_equals_simulator_exhaustive(P, S, W):
    """Every sequence of chunk sizes (in frames) up to 5 appends, incl. sink/window straddle and wrap."""
    frame_choices = [f for f in (1, 2, 3) if f * P <= W]
    for depth in (1, 2, 3, 4, 5):
        for seq in itertools.product(frame_choices, repeat=depth):
            c = RollingKVCache(S, W, P, width=3)
            for total in stream_chunks(c, [f * P for f in seq]):
                assert c.state() == closed_state(total, S, W), (seq, total)
                np.testing.assert_array_equal(c.slot_map(), closed_slot_map(total, S, W))


def test_sink_never_evicted_and_fifo_order():
    P, S, W = 4, 8, 12
    c = RollingKVCache(S, W, P, width=3)
    for total in stream_chunks(c, [4, 8, 4, 12, 4, 4, 8, 12, 4]):
        res = c.resident_ids()
        # the protected set is ids 0..S-1 for ever, in their own slots
        assert res[:min(total, S)] == list(range(min(total, S)))
        np.testing.assert_array_equal(c.slot_map()[:min(total, S)], np.arange(min(total, S)))
        # the window holds the most recent ids, contiguous and increasing
        win = res[min(total, S):]
        assert win == list(range(total - len(win), total))
        assert len(win) == min(max(total - S, 0), W)
    # tokens left in the order they arrived, and no sink token among them
    assert c.evicted_ids == list(range(S, S + len(c.evicted_ids)))
    assert len(c.evicted_ids) == c.total - S - W


def test_contents_follow_ids():
    P, S, W = 2, 2, 6
    c = RollingKVCache(S, W, P, width=3)
    for total in stream_chunks(c, [2, 4, 2, 6, 2]):
        k_phys, v_phys = c.slot_contents()
        for slot, gid in enumerate(c.slot_map()):
            if gid < 0:
                assert np.isnan(k_phys[slot]).all()
            else:
                kk, vv = rows([gid], 3)
                np.testing.assert_array_equal(k_phys[slot], kk[0])
                np.testing.assert_array_equal(v_phys[slot], vv[0])
        k, v = c.gather()
        kk, vv = rows(c.resident_ids(), 3)
        np.testing.assert_array_equal(k, kk)
        np.testing.assert_array_equal(v, vv)


def test_first_chunk_larger_than_sink_is_split():
    """A 3-frame first chunk with a 1-frame sink: frame 0 -> sink, frames 1-2 -> ring offsets 0-1."""
    P, S, W = 5, 5, 30
    c = RollingKVCache(S, W, P, width=3)
    sizes = [15, 15, 15, 15]
    totals = list(stream_chunks(c, sizes))
    assert totals[-1] == 60
    # ring offsets run 0-1, 2-4, then 5,0,1: the third chunk wraps in the middle of its append
    m = c.slot_map()
    np.testing.assert_array_equal(m[:5], np.arange(5))
    np.testing.assert_array_equal(m[5:15], np.arange(35, 45))     # ring frames 0,1 rewritten by chunk 2
    c2 = RollingKVCache(S, W, P, width=3)
    list(stream_chunks(c2, sizes[:3]))
    np.testing.assert_array_equal(c2.slot_map()[5 + 25:5 + 30], np.arange(30, 35))
    assert c2.state()["evicted"] == 45 - 5 - 30


def test_no_advance_overwrites_in_place():
    P, S, W = 2, 2, 4
    c = RollingKVCache(S, W, P, width=3)
    list(stream_chunks(c, [2, 2, 2, 2]))
    before_map = c.slot_map().copy()
    before_state = c.state()
    k, v = rows([100, 101], 3)
    c.append_evict(k, v, advance=False)
    np.testing.assert_array_equal(c.slot_map(), before_map)
    assert c.state() == before_state
    kk, vv = c.gather()
    np.testing.assert_array_equal(kk[-2:], k)
    np.testing.assert_array_equal(vv[-2:], v)
    # older residents untouched
    old_k, _ = rows(c.resident_ids()[:-2], 3)
    np.testing.assert_array_equal(kk[:-2], old_k)
    with pytest.raises(RuntimeError):
        c.append_evict(*rows([1, 2, 3, 4], 3), advance=False)


def test_argument_errors():
    with pytest.raises(ValueError):
        RollingKVCache(3, 4, 2, width=3)
    c = RollingKVCache(2, 4, 2, width=3)
    with pytest.raises(ValueError):
        c.append_evict(*rows(range(6), 3))        # larger than the window
    with pytest.raises(ValueError):
        c.append_evict(*rows(range(3), 3))        # not whole frames
    assert c.state()["total"] == 0


def test_reset():
    c = RollingKVCache(2, 4, 2, width=3)
    list(stream_chunks(c, [2, 4, 2]))
    c.reset()
    assert c.state() == closed_state(0, 2, 4)
    assert (c.slot_map() == -1).all()
