"""CPU oracle for the streaming causal video-DiT block and its rolling KV cache.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition that the
HIP library is checked against.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and
this package never imports the product.  It shares no code, table or helper
with the HIP library: everything here is numpy and Python containers.

What it follows (StreamDiffusionV2):
  * the streaming problem: short chunks per stream, each denoised in 1-4 steps
    (Section 1 "Efficiency objectives", Section 5.1 implementation details);
  * the sink-token-guided rolling KV cache with frame-by-frame updates
    (abstract; Section 1; Appendix D, rolling-KV-cache figure);
  * the adaptive sink refresh and the RoPE refresh (Section 4.1), in ``refresh.py``;
  * the motion-aware noise scheduler (Section 4.1), in ``motion.py``;
  * the SLO-aware batching scheduler (Section 4.1), in ``slo.py``;
  * the stream batch over denoising steps (Section 4.2), in ``stream_batch.py``;
  * latents in, latents out around the blocks (patch embedding, output head, few-step sampler update: none of them
    is in the paper, all are this build's readings), in ``latent_io.py``;
  * a causal DiT of the Wan 2.1 / CausVid lineage (Section 5.1 "Models") whose
    per-layer cost is 24 b L_q C^2 + 4 b L_q L_kv C (Appendix B).

The paper gives no block equations.  The block computed here is the reading
fixed by this build's design document (pre-norm adaLN block, q/k RMSNorm,
3D-RoPE, self-attention over the resident cache, text cross-attention, GELU
FFN).  Numerical agreement with the paper's trained model is therefore
"parity unpinned"; every function is pinned instead against library routines,
closed forms, invariants and brute force (tests/test_oracle_*.py).

Arithmetic is float64 by default; every entry point takes ``dtype`` so the
same code can run in float32 (a test bounds the difference).
"""

from .kv_cache import RollingKVCache  # noqa: F401
from .refresh import (  # noqa: F401
    sink_similarity,
    refresh_sink,
    adaptive_sink_update,
    rope_refresh_frame,
    rotate_keys,
)
from .slo import latency_model, frequency, pick_batch  # noqa: F401
from .stream_batch import StreamBatch  # noqa: F401
from .latent_io import (  # noqa: F401
    patchify,
    unpatchify,
    patch_embed,
    output_head,
    noise_latents,
    sampler_update,
    denoise_latents_step,
)
from .motion import (  # noqa: F401
    motion_intensity,
    normalized_motion,
    noise_rate,
    MotionNoiseScheduler,
)
from .dit_block import (  # noqa: F401
    layer_norm,
    rms_norm,
    gelu_tanh,
    silu,
    rope_3d,
    rope_pair_split,
    attention_dense,
    text_kv_prepare,
    dit_block_forward,
    timestep_embedding,
    timestep_vector,
    conditioning,
    denoise_step,
)
