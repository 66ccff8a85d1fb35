"""MI355X-native streaming causal video-DiT block with a sink + rolling KV cache.

The compute lives in ``libsdv2.so`` (hand-written HIP for gfx950, C ABI declared
in ``include/sdv2.h``); ``binding`` marshals torch device pointers into it.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""

__all__ = ["workloads", "cost_model", "binding", "runner"]
