"""Oracle of the sink-token-guided rolling KV cache (TEST INFRASTRUCTURE ONLY).

Follows the paper's description of the cache (abstract; Section 1; Appendix D,
rolling-KV-cache figure): a protected set of sink tokens plus a rolling window
of the most recent frames, updated frame by frame.  Readings the paper leaves
open and this build fixes:
  * the sink is the first ``S`` tokens of the stream and is never replaced;
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
        self.total = 0                     # tokens ever appended
        self.evicted_ids = []              # in the order they were dropped
        self.last_append = []              # ids written by the latest advancing append
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
            if len(self.last_append) != n:
                raise RuntimeError("advance=False needs a previous append of the same size")
            for row, gid in enumerate(self.last_append):
                self.values[gid] = (k[row].copy(), v[row].copy())
            return
        self.last_append = []
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

    def gather(self):
        """K and V of the resident tokens, in ``resident_ids()`` order."""
        ids = self.resident_ids()
        if not ids:
            z = np.zeros((0, self.width), dtype=self.dtype)
            return z, z.copy()
        k = np.stack([self.values[g][0] for g in ids])
        v = np.stack([self.values[g][1] for g in ids])
        return k, v

    def slot_map(self):
        """Token id held by each physical slot, -1 where nothing was written."""
        return np.asarray(self.slot_ids, dtype=np.int64)

    def slot_contents(self):
        """Physical image of the buffers: K and V ``[S+W, width]``; NaN where empty."""
        k = np.full((self.S + self.W, self.width), np.nan, dtype=self.dtype)
        v = np.full((self.S + self.W, self.width), np.nan, dtype=self.dtype)
        for slot, gid in enumerate(self.slot_ids):
            if gid >= 0:
                k[slot], v[slot] = self.values[gid]
        return k, v

    def state(self):
        """Counters compared bit for bit with the library's host-side state."""
        win_fill = len(self.window_ids)
        if win_fill:
            oldest_slot = self.slot_ids.index(self.window_ids[0])
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
