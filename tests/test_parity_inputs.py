"""What the GPU parity tests' inputs can and cannot resolve, shown with the oracle alone (CPU only).

The block output is x + three branch outputs.  With the seeded N(0, 0.02^2) modulation table the gates are
about 0.03, and the self-attention branch is a fraction of a percent of max |x|: a comparison of x_out at
2e-2 of max |x_out| cannot see it.  The GPU tests therefore also run with the weight edits of
``parity_util`` (gates of order one; the self-attention branch alone).  This file checks, on those tests' own
inputs, that switching the self-attention branch off in the oracle (W_o = b_o = 0) moves the compared quantity
by at least five times the bar.
"""

import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import oracle
from paper_2511_07399_amd import workloads as wk
from parity_util import OracleRunner, branch_floor, self_attention_alone, visible_branches

TOL_X = 2e-2


def dead_self_attention(base_edit):
    def edit(w, layer=0):
        if base_edit is not None:
            base_edit(w, layer)
        w["W_o"] *= 0.0
        w["b_o"] *= 0.0
    return edit


def outputs(wl, edit, chunks, zero_rows=()):
    ora = OracleRunner(wl, n_layers=1, n_streams=1, edit=edit)
    outs = []
    for chunk in range(chunks):
        x = wk.chunk_input(wl, chunk).double().numpy()
        if wl.name == "tiny":                       # as in the GPU tests: the tiny workload feeds a timestep vector
            e0 = ora.conditioning(tvec=wk.timestep_vector(wl, chunk).double().numpy())
        else:
            e0 = ora.conditioning(timestep=wk.timestep(wl, chunk))
        for r in zero_rows:
            e0[r] = 0.0
        dbg = {}
        y = ora.block(0, x, e0, (0, chunk * wl.frames_per_chunk, wl.frames_per_chunk, 1), debug=dbg)
        outs.append((x, y, dbg))
    return outs


@pytest.mark.parametrize("name,chunks", [("tiny", 4), ("wan1.3b-block", 1)])
def test_seeded_gates_hide_the_self_attention_branch_and_the_edits_show_it(name, chunks):
    wl = wk.WORKLOADS[name]
    # plain seeded weights: the dead branch stays under (or at) the bar of the x_out comparison
    live = outputs(wl, None, chunks)
    dead = outputs(wl, dead_self_attention(None), chunks)
    moved_plain = max(np.abs(a[1] - b[1]).max() / np.abs(a[1]).max() for a, b in zip(live, dead))
    # gates of order one: the same switch moves x_out by at least five bars, and no branch hides
    live = outputs(wl, visible_branches(wl), chunks)
    dead = outputs(wl, dead_self_attention(visible_branches(wl)), chunks)
    moved_visible = min(np.abs(a[1] - b[1]).max() / np.abs(a[1]).max() for a, b in zip(live, dead))
    for _, y, dbg in live:
        assert branch_floor(dbg) >= 5 * TOL_X * np.abs(y).max()
    # the self-attention branch alone: the update is that branch and nothing else
    alone = outputs(wl, self_attention_alone, chunks, zero_rows=(2, 5))
    for x, y, dbg in alone:
        upd = y - x
        assert np.abs(upd).max() > 0
        assert np.abs(upd - dbg["upd_self"]).max() <= 1e-9 * np.abs(upd).max()
    print("%s: dead self-attention moves x_out by %.2e (seeded gates), %.2e (gates of order one)"
          % (name, moved_plain, moved_visible))
    assert moved_plain < 1.5 * TOL_X
    assert moved_visible >= 5 * TOL_X
