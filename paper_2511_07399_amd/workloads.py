"""Named workload shapes and the seeded synthetic-input generators.

This module holds no arithmetic of the method: it only names shapes and draws
random tensors.  Both the HIP library's tests/benchmark and the CPU oracle's
tests take their inputs from here, so that the two sides see the same values.
Every tensor is drawn with a seeded PyTorch generator and rounded once to
bf16; matrices are returned as bf16, vectors as fp32 holding bf16-exact values.

The shapes stand in for the paper's workloads (Wan-2.1-1.3B / 14B shaped causal
DiT at 512x512 and 480x832, Section 5.1 and Section 5.2): one latent frame is
(H/16) x (W/16) tokens after the /8 VAE and the 1x2x2 patch embedding, a chunk
is a few latent frames, the cache holds one sink frame plus a window of recent
frames (Appendix B uses L_kv = 6 L_q at 1 560 tokens per frame).  Values are
random; trained weights and the evaluation videos are not used.
"""

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    C: int                 # model width
    H: int                 # heads (head dim = C // H)
    F: int                 # FFN width
    grid_h: int            # token rows per latent frame
    grid_w: int            # token columns per latent frame
    frames_per_chunk: int
    sink_frames: int
    window_frames: int     # window capacity, current chunk included
    L_t: int               # text tokens
    B: int                 # independent streams batched in one call
    N: int                 # blocks
    steps: tuple           # denoising steps per chunk that the workload names
    chunks: int            # chunks streamed
    t_dim: int = 256       # width of the sinusoidal timestep embedding

    @property
    def D(self):
        return self.C // self.H

    @property
    def P(self):           # tokens per latent frame
        return self.grid_h * self.grid_w

    @property
    def L(self):           # query tokens per stream per chunk
        return self.frames_per_chunk * self.P

    @property
    def S(self):           # sink capacity in tokens
        return self.sink_frames * self.P

    @property
    def W(self):           # window capacity in tokens
        return self.window_frames * self.P

    def block_flops(self, L_kv=None):
        """Algorithmic flops of one block for B streams (projections, FFN, both attentions)."""
        L_kv = self.S + self.W if L_kv is None else L_kv
        rows = self.B * self.L
        gemm = 2 * rows * (6 * self.C * self.C + 2 * self.C * self.F)
        self_attn = 4 * rows * L_kv * self.C
        cross_attn = 4 * rows * self.L_t * self.C
        return gemm + self_attn + cross_attn


WORKLOADS = {
    w.name: w for w in (
        Workload("tiny", 512, 4, 2048, 8, 16, 1, 1, 2, 64, 1, 1, (1,), 6),
        Workload("wan1.3b-block", 1536, 12, 8960, 32, 32, 1, 1, 2, 512, 1, 1, (1,), 64),
        Workload("wan1.3b-step", 1536, 12, 8960, 32, 32, 1, 1, 2, 512, 1, 30, (1, 2, 4), 200),
        Workload("wan14b-step", 5120, 40, 13824, 32, 32, 1, 1, 2, 512, 1, 40, (1, 4), 8),
        Workload("wan14b-480p-b4", 5120, 40, 13824, 30, 52, 3, 1, 6, 512, 4, 40, (2,), 6),
    )
}

# tensor ids used in the per-(layer, tensor) seeds
_BLOCK_TENSORS = (
    # name, shape as a function of (C, F), kind
    ("W_q", lambda C, F: (C, C), "matrix"), ("b_q", lambda C, F: (C,), "bias"),
    ("W_k", lambda C, F: (C, C), "matrix"), ("b_k", lambda C, F: (C,), "bias"),
    ("W_v", lambda C, F: (C, C), "matrix"), ("b_v", lambda C, F: (C,), "bias"),
    ("g_q", lambda C, F: (C,), "gain"), ("g_k", lambda C, F: (C,), "gain"),
    ("W_o", lambda C, F: (C, C), "matrix"), ("b_o", lambda C, F: (C,), "bias"),
    ("mod_table", lambda C, F: (6, C), "bias"),
    ("ln3_gamma", lambda C, F: (C,), "gain"), ("ln3_beta", lambda C, F: (C,), "bias"),
    ("W_cq", lambda C, F: (C, C), "matrix"), ("b_cq", lambda C, F: (C,), "bias"),
    ("g_cq", lambda C, F: (C,), "gain"),
    ("W_ck", lambda C, F: (C, C), "matrix"), ("b_ck", lambda C, F: (C,), "bias"),
    ("g_ck", lambda C, F: (C,), "gain"),
    ("W_cv", lambda C, F: (C, C), "matrix"), ("b_cv", lambda C, F: (C,), "bias"),
    ("W_co", lambda C, F: (C, C), "matrix"), ("b_co", lambda C, F: (C,), "bias"),
    ("W_1", lambda C, F: (F, C), "matrix"), ("b_1", lambda C, F: (F,), "bias"),
    ("W_2", lambda C, F: (C, F), "matrix"), ("b_2", lambda C, F: (C,), "bias"),
)
BLOCK_TENSOR_NAMES = tuple(n for n, _, _ in _BLOCK_TENSORS)

MODEL_LAYER = 10_000        # pseudo layer index for the conditioning weights
STD_W = 0.02


def _seed(base_seed, layer, tensor_id):
    return base_seed * 1_000_003 + layer * 101 + tensor_id


def _draw(shape, kind, seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * STD_W
    if kind == "gain":
        t = t + 1.0
    t = t.to(torch.bfloat16)
    return t if kind == "matrix" else t.to(torch.float32)


def block_weights(wl, layer, base_seed=0, device="cpu"):
    """This layer's tensors: matrices ``[out, in]`` bf16, vectors fp32 (bf16-exact)."""
    return {
        name: _draw(shape(wl.C, wl.F), kind, _seed(base_seed, layer, tid), device)
        for tid, (name, shape, kind) in enumerate(_BLOCK_TENSORS)
    }


def model_weights(wl, base_seed=0, device="cpu"):
    """Conditioning weights shared by all layers (timestep MLP and modulation projection)."""
    C = wl.C
    spec = (("W_t1", (C, wl.t_dim), "matrix"), ("b_t1", (C,), "bias"),
            ("W_t2", (C, C), "matrix"), ("b_t2", (C,), "bias"),
            ("W_mod", (6 * C, C), "matrix"), ("b_mod", (6 * C,), "bias"))
    return {name: _draw(shape, kind, _seed(base_seed, MODEL_LAYER, tid), device)
            for tid, (name, shape, kind) in enumerate(spec)}


IO_LAYER = 10_001           # pseudo layer index for the patch-embedding and head weights
LATENT_CHANNELS = 16        # VAE latent channels; a token covers 2 x 2 latent positions (64 numbers)


def io_weights(wl, base_seed=0, device="cpu"):
    """Patch-embedding and output-head weights: matrices bf16 ``[out, in]``, vectors fp32 (bf16-exact)."""
    C, P = wl.C, 4 * LATENT_CHANNELS
    spec = (("W_pe", (C, P), "matrix"), ("b_pe", (C,), "bias"), ("head_table", (2, C), "bias"),
            ("W_head", (P, C), "matrix"), ("b_head", (P,), "bias"))
    return {name: _draw(shape, kind, _seed(base_seed, IO_LAYER, tid), device)
            for tid, (name, shape, kind) in enumerate(spec)}


def latent_chunk(wl, chunk, stream=0, base_seed=0, device="cpu", kind=0):
    """A latent chunk ``[16, frames, 2 grid_h, 2 grid_w]`` ~ N(0,1), fp32 holding bf16-exact values (kind 0: the clean
    input, 1, 2, ...: the noise drawn for denoising step kind - 1)."""
    return _normal((LATENT_CHANNELS, wl.frames_per_chunk, 2 * wl.grid_h, 2 * wl.grid_w),
                   base_seed * 1_000_003 + 600_000 + 7919 * chunk + 97 * kind + stream, device)


def _normal(shape, seed, device="cpu"):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16).to(torch.float32)


def chunk_input(wl, chunk, stream=0, base_seed=0, device="cpu"):
    """Hidden state ``[L, C]`` of one stream's chunk, N(0,1), fp32 holding bf16-exact values."""
    return _normal((wl.L, wl.C), base_seed * 1_000_003 + 500_000 + 7919 * chunk + stream, device)


def text_context(wl, stream=0, base_seed=0, device="cpu"):
    """Text tokens ``[L_t, C]`` of one stream's prompt, N(0,1), bf16-exact."""
    return _normal((wl.L_t, wl.C), base_seed * 1_000_003 + 400_000 + stream, device)


def timestep_vector(wl, chunk, step=0, stream=0, base_seed=0, device="cpu"):
    """A ``[C]`` timestep vector N(0,1) for workloads that feed it directly (the tiny one)."""
    return _normal((wl.C,), base_seed * 1_000_003 + 300_000 + 7919 * chunk + 31 * step + stream, device)


def timestep(wl, chunk, step=0, stream=0, base_seed=0):
    """A timestep drawn uniformly in [0, 1000), as a Python float (fp32-exact)."""
    g = torch.Generator()
    g.manual_seed(base_seed * 1_000_003 + 200_000 + 7919 * chunk + 31 * step + stream)
    return float((torch.rand((), generator=g, dtype=torch.float32) * 1000.0).item())


def to_numpy(tensors):
    """Host float64 copies of a dict of tensors (what the oracle consumes)."""
    return {k: v.detach().to("cpu", torch.float64).numpy() for k, v in tensors.items()}
