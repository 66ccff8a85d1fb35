"""Oracle of the sink-token-guided rolling KV cache (TEST INFRASTRUCTURE ONLY).

Follows the paper's description of the cache (abstract; Section 1; Appendix D,
rolling-KV-cache figure): a protected set of sink tokens plus a rolling window
of the most recent frames, updated frame by frame.  Readings the paper leaves
open and this build fixes:
  * the sink is the first ``S`` tokens of the stream; it is never evicted, and is replaced only by an
    explicit refresh (``replace_sink_frame``, used by ``oracle.refresh``);
  * the window is first-in-first-out by global token id;
  * a chunk is appended first and then attended to (the window capacity counts
    the current chunk, as in Appendix B's L_kv = 6 L_q);
  * a repeated denoising step of the same chunk (``advance=False``) overwrites
    the values of the most recent append and moves nothing.

This is written as a naive simulator on purpose: a Python list for the sink, a
deque for the window (evict from the front when over capacity), and beside it
a model of the physical buffer with a write cursor.  No modular closed form is
used anywhere here; the closed form is a theorem that the tests check against
this simulator.
"""

from collections import deque

import numpy as np


class RollingKVCache:
    """One (layer, stream) cache.  Capacities are in tokens."""

    def __init__(self, sink_tokens, window_tokens, tokens_per_frame, width, dtype=np.float64):
        if sink_tokens < 0 or window_tokens <= 0 or tokens_per_frame <= 0:
            raise ValueError("bad capacities")
        if sink_tokens % tokens_per_frame or window_tokens % tokens_per_frame:
            raise ValueError("capacities must be whole frames")
        self.S = int(sink_tokens)
        self.W = int(window_tokens)
        self.P = int(tokens_per_frame)
        self.width = int(width)
        self.dtype = dtype
        self.reset()

    def reset(self):
        # logical view: which token ids are protected, which are in the window
        self.sink_ids = []                 # grows to S entries, then frozen
        self.window_ids = deque()          # oldest at the left
        self.values = {}                   # token id -> (k_row, v_row)
        self.sink_copy = {}                # sink slot -> (k_row, v_row) of a refreshed sink (its own copy)
        self.total = 0                     # tokens ever appended
        self.evicted_ids = []              # in the order they were dropped
        self.last_append = []              # ids written by the latest advancing append
        self.sealed = False                # set by a sink refresh: no advance=False until the next append
        # physical view: one array of S+W slots and a cursor into the ring part
        self.slot_ids = [-1] * (self.S + self.W)
        self.ring_cursor = 0               # next ring offset to be written

    # ------------------------------------------------------------------ append
    def append_evict(self, k, v, advance=True):
        """Store ``k``/``v`` rows ``[n, width]`` for the chunk's tokens.

        advance=True : the rows are new tokens; the oldest window tokens that no
                       longer fit are evicted.
        advance=False: the rows replace the values of the latest append
                       (same token ids, same slots); nothing is evicted.
        """
        k = np.asarray(k, dtype=self.dtype)
        v = np.asarray(v, dtype=self.dtype)
        n = k.shape[0]
        if k.shape != (n, self.width) or v.shape != (n, self.width):
            raise ValueError("k/v must be [n, width]")
        if n <= 0 or n > self.W or n % self.P:
            raise ValueError("n_tokens must be whole frames and fit the window")
        if not advance:
            if len(self.last_append) != n or self.sealed:
                raise RuntimeError("advance=False needs a previous append of the same size, not yet closed by a refresh")
            for row, gid in enumerate(self.last_append):
                self.values[gid] = (k[row].copy(), v[row].copy())
            return
        self.last_append = []
        self.sealed = False
        for row in range(n):
            gid = self.total
            self.total += 1
            self.values[gid] = (k[row].copy(), v[row].copy())
            self.last_append.append(gid)
            if len(self.sink_ids) < self.S:
                # still filling the protected set: slot = position in the sink
                self.slot_ids[len(self.sink_ids)] = gid
                self.sink_ids.append(gid)
                continue
            # window token: takes the slot under the cursor; whoever sat there leaves
            slot = self.S + self.ring_cursor
            displaced = self.slot_ids[slot]
            self.window_ids.append(gid)
            if len(self.window_ids) > self.W:
                oldest = self.window_ids.popleft()
                # the ring must displace exactly the first-in token
                assert oldest == displaced, "ring cursor and FIFO order disagree"
                self.evicted_ids.append(oldest)
                del self.values[oldest]
            else:
                assert displaced == -1
            self.slot_ids[slot] = gid
            self.ring_cursor += 1
            if self.ring_cursor == self.W:
                self.ring_cursor = 0

    # ------------------------------------------------------------------- views
    def resident_ids(self):
        """Token ids attended to, sink first, then window oldest to newest."""
        return list(self.sink_ids) + list(self.window_ids)

    def _sink_rows(self):
        """(k_row, v_row) of each filled sink slot, in slot order."""
        return [self.sink_copy[slot] if slot in self.sink_copy else self.values[gid]
                for slot, gid in enumerate(self.sink_ids)]

    def gather(self):
        """K and V of the resident tokens, in ``resident_ids()`` order."""
        rows = self._sink_rows() + [self.values[g] for g in self.window_ids]
        if not rows:
            z = np.zeros((0, self.width), dtype=self.dtype)
            return z, z.copy()
        k = np.stack([r[0] for r in rows])
        v = np.stack([r[1] for r in rows])
        return k, v

    # ------------------------------------------------------------------- refresh support
    def frame_rows(self, frame_back=0):
        """Token ids and (k, v) rows of one frame of the latest append; ``frame_back = 0`` is its last frame."""
        n_frames = len(self.last_append) // self.P
        if not 0 <= frame_back < n_frames:
            raise ValueError("frame_back outside the latest append")
        first = len(self.last_append) - (frame_back + 1) * self.P
        ids = self.last_append[first:first + self.P]
        if ids[0] < self.S:                # whole frames: the frame is either all sink or all window
            raise RuntimeError("the frame was stored in the sink itself")
        return ids, [self.values[gid] for gid in ids]

    def sink_frame_rows(self, sink_frame):
        """(k, v) rows of sink frame ``sink_frame`` (slots ``sink_frame*P ..``); the frame must be filled."""
        lo, hi = sink_frame * self.P, (sink_frame + 1) * self.P
        if sink_frame < 0 or hi > len(self.sink_ids):
            raise ValueError("sink frame not filled")
        return self._sink_rows()[lo:hi]

    def replace_sink_frame(self, sink_frame, ids, rows):
        """Sink frame ``sink_frame`` now holds copies of ``rows`` and reports ``ids`` in the slot map."""
        lo, hi = sink_frame * self.P, (sink_frame + 1) * self.P
        if sink_frame < 0 or hi > len(self.sink_ids) or len(ids) != self.P or len(rows) != self.P:
            raise ValueError("bad sink frame or frame size")
        for j in range(self.P):
            old = self.sink_ids[lo + j]
            self.sink_copy[lo + j] = (rows[j][0].copy(), rows[j][1].copy())
            self.sink_ids[lo + j] = ids[j]
            self.slot_ids[lo + j] = ids[j]
            # the original sink token's values are no longer referenced by anything
            if old < self.S and old in self.values and old not in self.sink_ids:
                del self.values[old]
        # a refresh closes the chunk: its K/V can no longer be rewritten by a repeated denoising step
        self.sealed = True

    def map_keys(self, fn):
        """Replace the K row of every resident entry by ``fn(k_row)`` (used by the RoPE refresh)."""
        for slot in list(self.sink_copy):
            k, v = self.sink_copy[slot]
            self.sink_copy[slot] = (fn(k), v)
        for gid in list(self.values):
            k, v = self.values[gid]
            self.values[gid] = (fn(k), v)

    def slot_map(self):
        """Token id held by each physical slot, -1 where nothing was written."""
        return np.asarray(self.slot_ids, dtype=np.int64)

    def slot_contents(self):
        """Physical image of the buffers: K and V ``[S+W, width]``; NaN where empty."""
        k = np.full((self.S + self.W, self.width), np.nan, dtype=self.dtype)
        v = np.full((self.S + self.W, self.width), np.nan, dtype=self.dtype)
        for slot, gid in enumerate(self.slot_ids):
            if gid >= 0:
                k[slot], v[slot] = self.sink_copy[slot] if slot in self.sink_copy else self.values[gid]
        return k, v

    def state(self):
        """Counters compared bit for bit with the library's host-side state."""
        win_fill = len(self.window_ids)
        if win_fill:
            oldest_slot = self.slot_ids.index(self.window_ids[0], self.S)    # the window copy: a refreshed sink may hold the id too
        else:
            oldest_slot = -1
        if len(self.sink_ids) < self.S:
            next_slot = len(self.sink_ids)
        else:
            next_slot = self.S + self.ring_cursor
        return {
            "total": self.total,
            "sink_fill": len(self.sink_ids),
            "win_fill": win_fill,
            "oldest_slot": oldest_slot,
            "next_slot": next_slot,
            "evicted": len(self.evicted_ids),
        }
