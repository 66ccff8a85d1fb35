"""Oracle of the stream batch over denoising steps (TEST INFRASTRUCTURE ONLY).

What the paper states (Section 1, contribution (1); Section 4.2 with the pipeline-parallel
stream-batch figure; Section 5.4 "Effectiveness of Stream Batch"):
  * the input is reformulated as a batch of B short chunks, and the n denoising steps of a
    chunk act as a batch multiplier: the latency model becomes L(T, n B);
  * the batch rows are latent streams at different noise levels ("depth" in the figure);
  * a fine-denoised (clean) latent leaves the batch at every micro-step;
  * more denoising steps mean a deeper pipeline of in-flight chunks.

Reading taken here (the paper prints no schedule and does not say what the rows share):
a stream that is denoised in n steps keeps n chunks in flight.  At every micro-step the
newest chunk enters at depth 0, every in-flight chunk makes ONE denoising step at its
current depth d with the timestep of that depth, all of them in one batched forward, and
the chunk that has just finished depth n - 1 leaves.  Each depth has its own rolling KV
cache: the keys and values a chunk writes at depth d are the history that the following
chunks read at depth d (the rows are "distinct latent streams", one per noise level).  A
chunk therefore goes through depths 0 .. n-1 in order, one micro-step each, and chunk c
leaves at micro-step c + n - 1.

This module holds only the schedule, written as the plain simulation of the statement
above: a list of in-flight chunks, no row indices, no modular arithmetic.  What one
denoising step at a depth computes is passed in as ``step_fn`` (the tests pass the
oracle's ``denoise_step`` on that depth's caches).
"""


class StreamBatch:
    """In-flight chunks of one stream that is denoised in ``n_steps`` steps per chunk.

    step_fn(x, depth, meta) -> x'   one denoising step of the chunk ``meta`` at noise depth
                                    ``depth`` (0 = noisiest); it owns whatever state the
                                    depth has (its caches).
    """

    def __init__(self, n_steps, step_fn):
        if n_steps < 1:
            raise ValueError("n_steps must be at least 1")
        self.n_steps = n_steps
        self.step_fn = step_fn
        self.in_flight = []          # oldest first: dicts with x, depth, meta
        self.micro_steps = 0

    def micro_step(self, x_new=None, meta=None):
        """One micro-step.  ``x_new`` is the chunk that enters (None: nothing enters, the pipeline
        drains).  Returns (rows, finished): the number of batch rows of this micro-step and the
        (meta, x) of the chunk that left, or None."""
        if x_new is not None:
            self.in_flight.append({"x": x_new, "depth": 0, "meta": meta})
        rows = len(self.in_flight)
        # one batched forward: every in-flight chunk makes one step at its own depth (the depths
        # are all different, and each depth has its own state, so the order does not matter)
        for item in self.in_flight:
            item["x"] = self.step_fn(item["x"], item["depth"], item["meta"])
            item["depth"] += 1
        finished = None
        if self.in_flight and self.in_flight[0]["depth"] == self.n_steps:
            done = self.in_flight.pop(0)
            finished = (done["meta"], done["x"])
        self.micro_steps += 1
        return rows, finished
