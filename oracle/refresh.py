"""Oracle of the adaptive sink refresh and the RoPE refresh (TEST INFRASTRUCTURE ONLY).

StreamDiffusionV2, Section 4.1, "Adaptive sink and RoPE refresh":
  * sinks S_t = {s_1 .. s_m}; with a new chunk embedding h_t,  alpha_i = cos(h_t, s_i);  a sink whose alpha_i is
    below the threshold tau is replaced by h_t, the others are kept;
  * once the frame index t exceeds T_reset the rotary phase of frame t is that of frame t - T_reset.

Readings fixed by this build where the section is silent (one object per (layer, stream) cache):
  * a sink s_i is one sink *frame* of the cache (tokens_per_frame tokens; m = sink_tokens / tokens_per_frame), and
    h_t is one frame of the chunk just appended (``frame_back = 0``: its last frame), so that "s_i = h_t" is a copy
    of that frame's cached K and V rows into the sink frame's slots;
  * the cosine is taken over the frames' *value* rows flattened to one vector of tokens_per_frame * C numbers:
    values carry no rotary phase, cached keys of different frames differ by their phases even for equal content;
  * the copied keys keep the rotary phase of the frame they came from, and the slot map reports the copied tokens'
    ids in the sink slots (until the source frame leaves the window the tokens are resident twice);
  * a refresh closes the chunk (no repeated denoising step may rewrite it afterwards);
  * cached keys are moved along with a RoPE reset: a key cached at frame f becomes the key of frame f - delta
    (its frame pairs turned by -delta * omega_j), so that every query/key phase *difference* is what it was.

No function here is pinned to a number printed in the paper (it prints none for these mechanisms): parity with the
paper is unpinned; the pins are closed forms and invariances (tests/test_oracle_refresh.py).
"""

import numpy as np

from .dit_block import rope_3d


def _flat_values(rows):
    return np.concatenate([np.asarray(r[1], dtype=np.float64) for r in rows])


def cosine(a, b):
    """cos(a, b) = <a, b> / (|a| |b|); 0 when either vector is zero."""
    na = float(np.sqrt(np.dot(a, a)))
    nb = float(np.sqrt(np.dot(b, b)))
    if na == 0.0 or nb == 0.0:
        return 0.0
    return float(np.dot(a, b) / (na * nb))


def sink_similarity(cache, frame_back=0):
    """alpha_i = cos(h_t, s_i) for every sink frame i (Section 4.1); h_t = frame ``frame_back`` of the latest append."""
    _, rows = cache.frame_rows(frame_back)
    h = _flat_values(rows)
    m = cache.S // cache.P
    return np.array([cosine(h, _flat_values(cache.sink_frame_rows(i))) for i in range(m)], dtype=np.float64)


def refresh_sink(cache, sink_frame, frame_back=0):
    """s_i <- h_t: sink frame ``sink_frame`` becomes a copy of frame ``frame_back`` of the latest append."""
    ids, rows = cache.frame_rows(frame_back)
    cache.replace_sink_frame(sink_frame, ids, rows)


def adaptive_sink_update(cache, tau, frame_back=0):
    """One update of the sink set (Section 4.1): keep s_i when alpha_i >= tau, else replace it by h_t.

    Returns (alpha, replaced) with ``replaced`` the list of refreshed sink frames."""
    alpha = sink_similarity(cache, frame_back)
    replaced = [i for i in range(len(alpha)) if not alpha[i] >= tau]
    for i in replaced:
        refresh_sink(cache, i, frame_back)
    return alpha, replaced


def rope_refresh_frame(t, t_reset):
    """Frame index whose rotary phase frame t uses (Section 4.1): t up to T_reset, t - T_reset beyond."""
    return t if t <= t_reset else t - t_reset


def rotate_keys(cache, delta_frames, n_heads):
    """Move every cached key ``delta_frames`` frames back in rotary phase (frame pairs turned by -delta * omega_j)."""
    D = cache.width // n_heads
    pos = np.array([[-delta_frames, 0, 0]], dtype=np.float64)

    def turn(k_row):
        return rope_3d(np.asarray(k_row, dtype=cache.dtype).reshape(1, n_heads, D), pos, cache.dtype).reshape(-1)

    cache.map_keys(turn)
