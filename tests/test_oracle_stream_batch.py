"""Pins of the stream-batch schedule oracle (CPU only).

The schedule is checked against what the paper states about it (Section 4.2 and its figure: the n denoising steps
multiply the batch; a clean latent leaves at every micro-step; more steps mean a deeper pipeline) and against the
de-pipelined definition: because every depth has its own caches and sees the chunks in stream order, the pipeline
must give, chunk for chunk, exactly what n nested sequential denoising steps per chunk give.
"""

import numpy as np
import pytest

import oracle
from paper_2511_07399_amd import workloads as wk


def make_depth_model(wl, n_steps, n_layers):
    """Per-depth caches of a small model and the step function that runs the oracle's denoise step on them."""
    layers = [wk.to_numpy(wk.block_weights(wl, layer)) for layer in range(n_layers)]
    mw = wk.to_numpy(wk.model_weights(wl))
    ctx = wk.text_context(wl).double().numpy()
    text = [oracle.text_kv_prepare(ctx, w) for w in layers]
    caches = [[oracle.RollingKVCache(wl.S, wl.W, wl.P, wl.C) for _ in range(n_layers)] for _ in range(n_steps)]

    def step_fn(x, depth, chunk):
        return oracle.denoise_step(x, mw, layers, caches[depth], [t[0] for t in text], [t[1] for t in text], wl.H,
                                   wl.P, wl.grid_w, chunk * wl.frames_per_chunk, advance=True,
                                   t=wk.timestep(wl, chunk, depth))
    return step_fn, caches


@pytest.mark.parametrize("n_steps", [1, 2, 4])
def test_schedule_counts_rows_and_emits_one_chunk_per_micro_step(n_steps):
    trace = []
    sb = oracle.StreamBatch(n_steps, lambda x, depth, meta: trace.append((meta, depth)) or x + 1)
    n_chunks = 7
    emitted = []
    for m in range(n_chunks + n_steps - 1):
        entering = m < n_chunks
        rows, fin = sb.micro_step(0 if entering else None, m if entering else None)
        # warm-up: the batch fills one row per micro-step; steady state: n rows (the batch multiplier); drain
        assert rows == min(m + 1, n_steps, n_chunks + n_steps - 1 - m)
        if fin is not None:
            emitted.append((m, fin[0], fin[1]))
    # chunk c leaves at micro-step c + n - 1, after exactly n steps, and from then on one chunk per micro-step
    assert [(m, c) for m, c, _ in emitted] == [(c + n_steps - 1, c) for c in range(n_chunks)]
    assert all(x == n_steps for _, _, x in emitted)
    # every chunk went through depths 0 .. n-1 in order, and every depth saw the chunks in stream order
    for c in range(n_chunks):
        assert [d for meta, d in trace if meta == c] == list(range(n_steps))
    for d in range(n_steps):
        assert [meta for meta, dd in trace if dd == d] == list(range(n_chunks))


def test_one_step_per_chunk_is_plain_streaming():
    sb = oracle.StreamBatch(1, lambda x, depth, meta: x * 2)
    for c in range(4):
        rows, fin = sb.micro_step(float(c), c)
        assert rows == 1 and fin == (c, 2.0 * c)
    assert sb.micro_step() == (0, None)


@pytest.mark.parametrize("n_steps", [2, 3])
def test_pipeline_equals_nested_sequential_steps(n_steps):
    """The pipelined schedule against its definition without a pipeline: for each chunk in stream order, n denoising
    steps in a row, step d on the caches of depth d.  Bit-identical: the same calls reach every cache in the same
    order.  The model is a two-block version of the tiny workload, six chunks, so the depth caches evict."""
    wl = wk.WORKLOADS["tiny"]
    n_layers, n_chunks = 2, 6
    xs = [wk.chunk_input(wl, c).double().numpy() for c in range(n_chunks)]
    step_a, caches_a = make_depth_model(wl, n_steps, n_layers)
    sb = oracle.StreamBatch(n_steps, step_a)
    piped = {}
    for m in range(n_chunks + n_steps - 1):
        _, fin = sb.micro_step(xs[m] if m < n_chunks else None, m if m < n_chunks else None)
        if fin is not None:
            piped[fin[0]] = fin[1]
    step_b, caches_b = make_depth_model(wl, n_steps, n_layers)
    for c in range(n_chunks):
        x = xs[c]
        for d in range(n_steps):
            x = step_b(x, d, c)
        assert np.array_equal(piped[c], x), c
    for d in range(n_steps):
        for layer in range(n_layers):
            assert caches_a[d][layer].state() == caches_b[d][layer].state()
            assert caches_a[d][layer].state()["evicted"] > 0
            assert np.array_equal(caches_a[d][layer].slot_map(), caches_b[d][layer].slot_map())
    # and the depths really differ: the chunk's hidden state changes from step to step
    assert not np.array_equal(piped[0], step_b(xs[0], 0, 0))
