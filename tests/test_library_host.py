"""Host-side checks that need no GPU: the built library loads, exports every symbol the header
declares, sizes its buffers as documented and rejects bad arguments before touching anything."""

import ctypes as C
import os
import re

import pytest

from paper_2511_07399_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "sdv2.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sdv2_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 20
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.sdv2_version() >= 1


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(binding.ModelCfg) == 44
    assert C.sizeof(binding.CacheCfg) == 28
    assert C.sizeof(binding.ChunkDesc) == 16
    assert C.sizeof(binding.CacheState) == 32
    assert C.sizeof(binding.BlockWeights) == 8 + 23 * 8
    assert C.sizeof(binding.ModelWeights) == 8 + 7 * 8


def test_cache_bytes_formula(lib):
    # per (layer, stream): K and V^T of n_heads * cap * 128 bf16 each, plus cap int64 ids; cap = 64-aligned S+W
    cfg = binding.cache_cfg(30, 1, 12, 1024, 1024, 2048)
    cap = 3072
    assert binding.kv_cache_bytes(cfg) == 30 * (2 * 12 * cap * 128 * 2 + cap * 8)
    cfg = binding.cache_cfg(2, 4, 40, 1560, 1560, 9360)
    cap = 10944                                   # 10920 rounded up to 64
    assert binding.kv_cache_bytes(cfg) == 8 * (2 * 40 * cap * 128 * 2 + cap * 8)


@pytest.mark.parametrize("args", [
    (1, 1, 1, 4, -4, 8),      # negative sink
    (1, 1, 1, 4, 4, 0),       # empty window
    (1, 1, 1, 4, 6, 8),       # sink not whole frames
    (1, 1, 1, 4, 4, 10),      # window not whole frames
    (0, 1, 1, 4, 4, 8),       # no layers
])
def test_cache_cfg_errors(lib, args):
    with pytest.raises(binding.Sdv2Error) as e:
        binding.kv_cache_bytes(binding.cache_cfg(*args))
    assert e.value.code == binding.INVALID_ARG


def test_empty_cache_state_and_init_errors(lib):
    cfg = binding.cache_cfg(2, 3, 1, 4, 4, 8)
    need = lib.sdv2_kv_cache_bytes(C.byref(cfg))
    h = C.c_void_p()
    fake = C.c_void_p(0x10000)                    # never dereferenced: init launches nothing
    assert lib.sdv2_kv_cache_init(C.byref(cfg), fake, need - 1, C.byref(h)) == binding.INVALID_ARG
    assert lib.sdv2_kv_cache_init(C.byref(cfg), None, need, C.byref(h)) == binding.INVALID_ARG
    assert lib.sdv2_kv_cache_init(C.byref(cfg), C.c_void_p(0x10010), need, C.byref(h)) == binding.INVALID_ARG
    assert lib.sdv2_kv_cache_init(C.byref(cfg), fake, need, C.byref(h)) == binding.OK
    st = binding.kv_cache_state(h, 1, 2)
    assert st == {"total": 0, "sink_fill": 0, "win_fill": 0, "oldest_slot": -1, "next_slot": 0, "evicted": 0}
    assert binding.kv_cache_slot_map(h, 1, 2, 12) == [-1] * 12
    with pytest.raises(binding.Sdv2Error):
        binding.kv_cache_state(h, 2, 0)
    with pytest.raises(binding.Sdv2Error):
        binding.kv_cache_state(h, 0, 3)
    binding.kv_cache_destroy(h)


def test_workspace_sizes_and_model_cfg_errors(lib):
    cfg = binding.model_cfg(1536, 12, 8960, 32, 32, 512, 30)
    rows, Cw, F = 1024, 1536, 8960
    # h, qkv, q, o, u in bf16 at least
    assert binding.block_workspace_bytes(cfg, 1, 1024) >= rows * (6 * Cw + F) * 2
    assert binding.denoise_workspace_bytes(cfg, 1, 1024) > binding.block_workspace_bytes(cfg, 1, 1024)
    assert binding.text_kv_bytes(cfg) == 512 * 1536 * 2
    bad = binding.model_cfg(1500, 12, 8960, 32, 32, 512, 30)
    assert binding.block_workspace_bytes(bad, 1, 1024) == 0
    assert binding.block_workspace_bytes(cfg, 9, 1024) == 0          # more streams than SDV2_MAX_BATCH


def test_slo_pick_batch_matches_the_oracle_on_random_tables():
    """Host-only entry point: the library's choice of B* against the oracle's on 500 random latency tables."""
    import numpy as np
    import oracle
    binding.load_library()
    g = np.random.default_rng(1)
    for trial in range(500):
        sizes = g.permutation(g.choice(np.arange(1, 20), size=int(g.integers(1, 7)), replace=False)).tolist()
        lat = {int(B): float(g.uniform(0.5, 3.0)) * (0.3 + B) * 1e-3 for B in sizes}
        T = int(g.integers(1, 5))
        f_slo = float(g.uniform(100, 3000))
        frames = int(g.integers(0, 60))
        tol = float(g.choice([0.0, 0.05, 0.2]))
        got = binding.slo_pick_batch(lat, T, f_slo, frames, tol)
        want = oracle.pick_batch(lat, T, f_slo, frames, tol)
        if want is None:
            assert got is None
        else:
            assert got[0] == want[0] and got[2] == want[2] and abs(got[1] - want[1]) <= 1e-9 * want[1]
    for bad in (lambda: binding.slo_pick_batch({0: 1.0}, 1, 1.0, 10), lambda: binding.slo_pick_batch({1: 0.0}, 1, 1.0, 10),
                lambda: binding.slo_pick_batch({1: 1.0}, 0, 1.0, 10), lambda: binding.slo_pick_batch({1: 1.0}, 1, 1.0, 10, 1.0)):
        try:
            bad()
            assert False, "accepted a bad argument"
        except binding.Sdv2Error as e:
            assert e.code == binding.INVALID_ARG


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU only: bench.py --gpus N with N > 1 says so and exits without touching a GPU."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_stream_batch_handle_and_planner_hooks_on_the_host(lib):
    """Host-only parts of the newer entry points: stream-batch handle validation (nothing is launched), the planner's
    kernel names, and the tuning hook's parsing."""
    cfg = binding.model_cfg(512, 4, 2048, 8, 16, 64, 1)
    need = binding.stream_batch_rows_bytes(cfg, 4, 1)
    assert need >= 4 * 128 * 512 * 4
    assert binding.stream_batch_rows_bytes(cfg, 9, 1) == 0            # more depths than SDV2_MAX_BATCH
    fake = C.c_void_p(0x100000)                                       # never dereferenced by create
    h = C.c_void_p()
    ids = (C.c_int32 * 4)(0, 1, 2, 3)
    same = (C.c_int32 * 4)(0, 1, 1, 3)
    f = lib.sdv2_stream_batch_create
    assert f(C.byref(cfg), 4, same, 1, fake, need, C.byref(h)) == binding.INVALID_ARG
    assert f(C.byref(cfg), 4, ids, 1, fake, need - 256, C.byref(h)) == binding.WORKSPACE_TOO_SMALL
    assert f(C.byref(cfg), 4, ids, 1, C.c_void_p(0x100010), need, C.byref(h)) == binding.INVALID_ARG     # alignment
    assert f(C.byref(cfg), 0, ids, 1, fake, need, C.byref(h)) == binding.INVALID_ARG
    assert f(C.byref(cfg), 4, ids, 1, fake, need, C.byref(h)) == binding.OK
    assert lib.sdv2_stream_batch_reset(h) == binding.OK
    assert lib.sdv2_stream_batch_destroy(h) == binding.OK
    assert lib.sdv2_denoise_graph_state_bytes() >= 8 * (8 + 4 + 4 + 4)
    # the planner's kernel names: large shapes take the 256 x 256 alternating kernel, the single-chunk attention of the 1.3B
    # block the key-split form, a capacity that is no multiple of 128 the one-key-stream form
    assert binding.prof_kernel_name("gemm", 4, 4680, 13824, 5120, 1).startswith("gemm_alt64_kernel<")
    # an activation matrix of 4 GiB or more is beyond the 32-bit lane offsets of the direct-load kernels
    assert binding.prof_kernel_name("gemm", 8, 40000, 8192, 8192, 0).startswith("gemm_kernel<")
    assert binding.prof_kernel_name("gemm", 8, 30000, 8192, 8192, 0).startswith("gemm_alt64_kernel<")
    assert binding.prof_kernel_name("attention", 1, 1024, 12, 3072, 3072) == "attention_ks_kernel<2, 4>"
    assert binding.prof_kernel_name("attention", 1, 1024, 12, 3072, 3136).startswith("attention_kernel<")
    assert binding.prof_kernel_name("attention", 4, 4680, 40, 10920, 10944) == "attention_kernel<8>"
    binding.tuning_set("gemm_tile", "1,3")
    try:
        assert binding.prof_kernel_name("gemm", 4, 4680, 13824, 5120, 1) == "gemm_kernel<1, 3, 64, 2>"
    finally:
        binding.tuning_set("gemm_tile", None)
    for name, value in (("gemm_tile", "9,9"), ("attn_waves", "3"), ("no_such_knob", "1")):
        with pytest.raises(binding.Sdv2Error) as e:
            binding.tuning_set(name, value)
        assert e.value.code == binding.INVALID_ARG
    assert binding.gemm_noalloc_max_scratch_bytes() == 32 << 20


def test_latent_io_sizes_and_refusals_on_the_host(lib):
    """Host-only parts of the latents-in / latents-out entry points: workspace sizes and the argument checks that
    come before any launch (nothing here touches a GPU)."""
    cfg = binding.model_cfg(512, 4, 2048, 8, 16, 64, 2)
    L = 8 * 16
    io_ws = binding.latent_io_workspace_bytes(cfg, 3, L)
    assert io_ws >= 3 * L * 512 * 2 + 3 * L * 64 * 4 and io_ws % 256 == 0
    assert binding.latent_io_workspace_bytes(cfg, 0, L) == 0 and binding.latent_io_workspace_bytes(cfg, 9, L) == 0
    total = binding.denoise_latents_workspace_bytes(cfg, 3, L)
    assert total >= binding.denoise_workspace_bytes(cfg, 3, L) + io_ws + 3 * L * 512 * 4
    fake = C.c_void_p(0x100000)                                       # never dereferenced: every call below is refused
    one = (C.c_float * 1)(0.5)
    big = (C.c_float * 1)(1.5)
    less = (C.c_float * 1)(0.25)
    assert lib.sdv2_noise_latents(None, fake, fake, 1, 1024, one, None) == binding.INVALID_ARG
    assert lib.sdv2_noise_latents(fake, fake, fake, 1, 1024, big, None) == binding.INVALID_ARG          # rate above 1
    assert lib.sdv2_noise_latents(fake, fake, fake, 9, 1024, one, None) == binding.INVALID_ARG          # too many streams
    assert lib.sdv2_sampler_update(fake, fake, fake, fake, None, 1, 1024, less, one, None) == binding.INVALID_ARG   # sigma grows
    assert lib.sdv2_sampler_update(fake, fake, None, fake, None, 1, 1024, one, less, None) == binding.INVALID_ARG   # noise missing
    assert lib.sdv2_sampler_update(fake, fake, fake, fake, None, 1, 0, one, less, None) == binding.INVALID_ARG
    io = binding.IoWeights()                                          # struct_size 0, null pointers
    assert lib.sdv2_patch_embed(C.byref(cfg), C.byref(io), fake, 1, 1, fake, fake, io_ws, None) == binding.INVALID_ARG
    assert lib.sdv2_output_head(C.byref(cfg), C.byref(io), fake, fake, 1, 1, fake, fake, io_ws, None) == binding.INVALID_ARG
    assert b"io weights" in lib.sdv2_last_error()
    assert lib.sdv2_prof_lds_rates(100, None, 40960, None) == binding.INVALID_ARG
    assert lib.sdv2_prof_lds_rates(100, fake, 1024, None) == binding.INVALID_ARG


def test_stream_batch_of_latents_sizes_on_the_host(lib):
    cfg = binding.model_cfg(512, 4, 2048, 8, 16, 64, 2)
    L = 8 * 16
    for n in (1, 2, 4):
        need = binding.stream_batch_latents_workspace_bytes(cfg, n, 1)
        assert need >= binding.denoise_latents_workspace_bytes(cfg, n, L) + n * 64 * L * 4
        # the rows buffer of the handle (hidden states) also holds the latent rows
        assert binding.stream_batch_rows_bytes(cfg, n, 1) >= n * 64 * L * 4
    assert binding.stream_batch_latents_workspace_bytes(cfg, 9, 1) == 0
