"""GPU parity of the individual kernels, through the C ABI, against the CPU oracle.

Tolerances: the dense kernels multiply bf16 operands exactly and accumulate in fp32, so against the
float64 oracle on the same bf16 inputs the only errors are fp32 summation order (relative 1e-6 per
term) and the final rounding of the output to bf16 (relative 2^-9).  Attention also rounds the
probabilities to bf16 before the second product.  Bars: 1e-2 of the largest output for bf16 outputs,
1e-4 for fp32 outputs; cache bookkeeping and copied cache contents are bit-exact.
"""


import math
import numpy as np
import pytest
import torch

import oracle
from oracle.dit_block import linear as oracle_linear
from paper_2511_07399_amd import binding
from parity_util import max_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16_randn(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


# ------------------------------------------------------------------------------------------ GEMM
GEMM_CASES = [
    # M, N, K, epilogue, tile override ("tm,tn[,pf[,parts of k]]" register-staged kernel, "d<id>" direct-load kernel) or None
    (128, 128, 64, 0, None),
    (1, 128, 64, 0, None),                 # a single row
    (200, 384, 192, 0, "1,3"),             # ragged M, N tile of 96
    (333, 640, 512, 1, "2,5"),             # GELU epilogue, 256 x 160 tiles, ragged M
    (1024, 1536, 512, 0, "1,7"),           # N not a multiple of the 224-wide tile
    (300, 512, 1024, 2, "1,4"),            # gated residual, ragged M
    (300, 512, 1024, 2, None),
    (260, 256, 2048, 3, "2,8"),            # residual, biggest tile
    (300, 384, 768, 0, "1,3,3"),           # three register sets (loads three k tiles ahead), 12 k tiles
    (520, 640, 704, 2, "2,5,3"),           # three sets, 11 k tiles (tail of the unrolled-by-6 loop)
    (256, 256, 64, 3, "2,2,3"),            # three sets, a single k tile
    (256, 384, 448, 1, "1,6,3"),           # three sets, 7 k tiles
    (1024, 2048, 512, 1, None),            # tiny workload FFN-1
    (1024, 4608, 1536, 0, None),           # 1.3B QKV
    (1024, 1536, 8960, 2, None),           # 1.3B FFN-2
    (1024, 15360, 5120, 0, None),          # 14B QKV: the planner picks the direct-load kernel
    (1000, 1536, 512, 0, "d1"),            # direct-load kernel, 256 x 256 tiles, ragged M
    (300, 640, 192, 3, "d2"),              # direct-load kernel, N not a multiple of the tile, 3 k tiles
    (256, 256, 64, 2, "d2"),               # a single k tile
    (520, 2048, 1024, 1, "d3"),            # 128 x 256 tiles, three LDS stages, GELU
    (128, 512, 512, 2, "d4"),              # 256 x 128 tiles, a single ragged M tile
    (260, 384, 128, 0, "d3"),              # two k tiles in a three-stage ring
    (1000, 1536, 512, 1, "d5"),            # ring of four k32 stages, GELU, ragged M
    (300, 640, 192, 2, "d6"),              # ring variant, N not a multiple of the tile, 6 k tiles
    (256, 256, 64, 3, "d6"),               # two k tiles: fewer than the ring holds
    (130, 256, 32 * 2, 0, "d5"),           # K = 64
    (520, 768, 1024, 2, "d6,3"),           # ring with three k parts (fp32 partial sums + reduce), gated residual
    (1000, 512, 640, 1, "d5,2"),           # ring, two k parts, GELU in the reduce pass, ragged M
    (1000, 1536, 512, 1, "d17"),           # two wave groups half a step apart, half stages of 64 k; GELU, ragged M
    (300, 640, 192, 2, "d18"),             # 3 k tiles, N not a multiple of the tile
    (256, 256, 64, 3, "d18"),              # one k tile
    (130, 256, 128, 0, "d17"),             # two k tiles
    (520, 768, 1024, 2, "d18,3"),          # three k parts
    (2048, 2048, 2048, 0, "d18"),          # 64 full tiles, 32 k tiles
    (1024, 1024, 320, 0, "d17"),           # five k tiles: one turn of the slot ring
    (1024, 1024, 384, 0, "d18"),           # six k tiles
    (300, 512, 1024, 2, "1,4,2,2"),        # k split in two parts + reduce kernel, gated residual, ragged M
    (260, 256, 2048, 3, "2,8,2,4"),        # four parts, residual
    (1024, 1536, 1536, 1, "1,5,2,3"),      # three parts, GELU in the reduce kernel, ragged N tile
    (130, 384, 192, 0, "1,3,2,8"),         # more parts asked than k allows: clamped to one part per two k tiles
    (300, 384, 320, 0, "d7"),              # small tiles of the direct-load kernel: 128 x 64, three stages, 5 k tiles
    (1024, 1536, 1536, 2, "d8"),           # 128 x 64, four stages: the C x C projections of the 1.3B block
    (200, 640, 192, 1, "d9"),              # 128 x 64 with eight waves of 32 x 32, 3 k tiles in a four-stage ring
    (260, 512, 448, 3, "d10"),             # 64 x 128
    (520, 768, 1024, 2, "d11,2"),          # 128 x 128 four waves, two k parts
    (333, 640, 512, 1, "d12"),             # 128 x 128 eight waves, ragged M and N
    (1024, 8960, 1536, 1, "d13"),          # 128 x 160 two stages: FFN-1 of the 1.3B block
    (300, 1280, 256, 0, "d14"),            # 128 x 160 three stages
    (130, 768, 640, 2, "d15,3"),           # 128 x 192, three k parts
    (1000, 1536, 512, 1, "d16"),           # 128 x 192 with eight waves of 32 x 96
    (1024, 1536, 8960, 2, "d15,4"),        # FFN-2 of the 1.3B block, four k parts
]


@pytest.mark.parametrize("M,N,K,epi,tile", GEMM_CASES)
def test_gemm_matches_oracle(M, N, K, epi, tile):
    a = bf16_randn((M, K), 1)
    w = bf16_randn((N, K), 2, 0.05)
    bias = bf16_randn((N,), 3, 0.5).float()
    rows_per_gate = max(M // 3, 1)
    n_gate = (M + rows_per_gate - 1) // rows_per_gate
    gate_a = bf16_randn((N,), 4, 0.3).float()
    gate_b = bf16_randn((n_gate, 2 * N), 5, 0.3).float()        # stride 2N: a strided table
    x0 = bf16_randn((M, N), 6).float()
    acc = oracle_linear(f64(a), f64(w), f64(bias))
    if epi == 0:
        want = acc
    elif epi == 1:
        want = oracle.gelu_tanh(acc)
    elif epi == 2:
        gate = f64(gate_a)[None, :] + f64(gate_b)[np.arange(M) // rows_per_gate, :N]
        want = f64(x0) + gate * acc
    else:
        want = f64(x0) + acc
    binding.tuning_set("gemm_tile", tile)
    try:
        # with the scratch the plan asks for (NaN-filled: every partial sum that is read was written), then without
        ws_bytes = binding.gemm_workspace_bytes(M, N, K, epi)
        ws = torch.full((ws_bytes // 4,), float("nan"), dtype=torch.float32, device=DEV) if ws_bytes else None
        for workspace in ([ws, None] if ws is not None else [None]):
            out = (torch.empty(M, N, dtype=torch.bfloat16) if epi < 2 else x0.clone()).to(DEV)
            binding.gemm_bf16(a.to(DEV), w.to(DEV), bias.to(DEV), out, epi, gate_a.to(DEV), gate_b.to(DEV), 2 * N,
                              rows_per_gate, workspace=workspace)
            torch.cuda.synchronize()
            err = max_rel_err(f64(out), want)
            assert err < (1e-2 if epi < 2 else 1e-4), err
    finally:
        binding.tuning_set("gemm_tile", None)


def test_gemm_full_size_batched_480p_shape_sampled_rows():
    """FFN-1 of the 14B-shaped block on 4 streams x 4680 tokens (M 18720, N 13824, K 5120: the direct-load kernel,
    74 x 54 tiles, ragged last M tile): whole output finite, 48 sampled rows against the oracle."""
    M, N, K = 18720, 13824, 5120
    g = torch.Generator(device=DEV).manual_seed(7)
    a = torch.randn(M, K, generator=g, device=DEV).to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g, device=DEV) * 0.02).to(torch.bfloat16)
    bias = (torch.randn(N, generator=g, device=DEV) * 0.5).to(torch.bfloat16).float()
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    binding.gemm_bf16(a, w, bias, out, 1)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rows = sorted(set(np.random.default_rng(0).integers(0, M, 44).tolist()) | {0, 255, 256, M - 1})
    want = oracle.gelu_tanh(oracle_linear(f64(a[rows]), f64(w), f64(bias)))
    assert max_rel_err(f64(out[rows]), want) < 1e-2


def test_gemm_rejects_bad_shapes():
    a = torch.zeros(8, 100, dtype=torch.bfloat16, device=DEV)
    w = torch.zeros(128, 100, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(8, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.Sdv2Error) as e:
        binding.gemm_bf16(a, w, None, out)
    assert e.value.code == binding.INVALID_ARG


# ------------------------------------------------------------------------------------------ attention
def pack_kv(k_rows, v_rows, H, cap):
    """Token rows [n, C] -> the cache layouts K [H][cap][128], V^T [H][128][cap] (slot s in column vt_columns[s]);
    padding slots are NaN."""
    n, Cw = k_rows.shape
    D = Cw // H
    K = torch.full((H, cap, D), float("nan"), dtype=torch.bfloat16)
    VT = torch.full((H, D, cap), float("nan"), dtype=torch.bfloat16)
    K[:, :n, :] = k_rows.reshape(n, H, D).permute(1, 0, 2)
    VT[:, :, binding.vt_columns(cap)[:n]] = v_rows.reshape(n, H, D).permute(1, 2, 0)
    return K.contiguous(), VT.contiguous()


ATTN_CASES = [
    # B, L, H, kv_lens, forced splits
    (1, 128, 1, [64], 0),
    (1, 32, 2, [1], 0),                    # a single key
    (1, 100, 2, [63], 0),                  # ragged queries and keys inside one tile
    (1, 130, 2, [65], 0),                  # one key into the second tile
    (2, 300, 3, [384, 129], 0),            # two streams with different lengths
    (1, 128, 4, [384], 3),                 # split-KV, merged
    (2, 200, 2, [1000, 70], 4),            # a stream with fewer tiles than splits
    (1, 1024, 12, [3072], 0),              # 1.3B steady state (planner's split)
    (1, 1024, 12, [512], 0),               # text cross-attention shape
    (1, 70, 2, [200], 0),                  # a 128-key tile and a tail of 72: slices 2 and 3 of the tail hold 8 and 0 keys
    (2, 64, 1, [40, 129], 0),              # fewer keys than one slice; one key into the second 128-key tile
]


# waves 0: the planner's choice; 4 / 8: 128 / 256 queries per workgroup, one key stream; 2: the key-split form
# (2 query blocks x 4 key slices per workgroup, 128-key tiles, capacity a multiple of 128)
@pytest.mark.parametrize("waves", [0, 4, 8, 2])
@pytest.mark.parametrize("B,L,H,kv_lens,splits", ATTN_CASES)
def test_attention_matches_oracle(B, L, H, kv_lens, splits, waves):
    D = 128
    Cw = H * D
    q = bf16_randn((B, L, Cw), 10)
    ks, vts, caps, want = [], [], [], []
    for b, n in enumerate(kv_lens):
        k_rows = bf16_randn((n, Cw), 20 + b)
        v_rows = bf16_randn((n, Cw), 30 + b)
        cap = (n + 127) // 128 * 128 + 128 * (b % 2) if waves == 2 else (n + 63) // 64 * 64 + 64 * (b % 2)
        K, VT = pack_kv(k_rows, v_rows, H, cap)
        ks.append(K.to(DEV))
        vts.append(VT.to(DEV))
        caps.append(cap)
        want.append(oracle.attention_dense(f64(q[b]).reshape(L, H, D), f64(k_rows).reshape(n, H, D),
                                           f64(v_rows).reshape(n, H, D)).reshape(L, Cw))
    o = torch.full((B, L, Cw), float("nan"), dtype=torch.bfloat16, device=DEV)
    binding.tuning_set("attn_splits", splits or None)
    binding.tuning_set("attn_waves", waves or None)
    try:
        ws = torch.empty(max(binding.attention_workspace_bytes(B, L, Cw, max(kv_lens)), 256), dtype=torch.uint8, device=DEV)
        binding.attention_bf16(q.to(DEV), ks, vts, kv_lens, caps, o, H, ws)
        torch.cuda.synchronize()
    finally:
        binding.tuning_set("attn_splits", None)
        binding.tuning_set("attn_waves", None)
    got = f64(o)
    assert np.isfinite(got).all()
    for b in range(B):
        err = max_rel_err(got[b], want[b])
        assert err < 1e-2, (b, err)


# Score profiles along the key index, in log2 units of the exponent (what the kernel's running reference point is
# measured in).  The kernels keep that reference only loosely behind the row maximum and form no maximum in the
# steady state, so these walk through every way the reference has to move: maxima that keep growing across tiles,
# one key far above everything seen, scores far above and far below zero from the first key on, maxima that only fall.
SCORE_PROFILES = {
    "growing": lambda j, n: 100.0 * j / n,
    "falling": lambda j, n: 100.0 * (1.0 - j / n),
    "spike": lambda j, n: np.where(j == n // 2 + 3, 200.0, 0.0),
    "huge": lambda j, n: 300.0 + 5.0 * np.sin(j),
    "far below zero": lambda j, n: -300.0 + 5.0 * np.sin(j),
    "steps": lambda j, n: 20.0 * (j // 90),
}


@pytest.mark.parametrize("waves,splits", [(0, 0), (4, 0), (8, 0), (2, 0), (4, 3)])
@pytest.mark.parametrize("profile", sorted(SCORE_PROFILES))
def test_attention_score_ranges(profile, waves, splits):
    """q_i = a_i u + noise, k_j = b_j u + noise with u in {-1, +1}^128, so that the scaled score of (i, j) in log2 units is
    about a_i T(j): a_i runs from 0.5 to 1.5 over the queries and is negated for every third query (its profile is
    mirrored), so the lanes of a wave need their reference moved at different tiles, and some never."""
    L, H, D, n = 96, 2, 128, 700
    Cw = H * D
    g = torch.Generator().manual_seed(77)
    u = (torch.randint(0, 2, (H, D), generator=g) * 2 - 1).to(torch.float32)
    per_unit = math.sqrt(D) * math.log2(math.e)          # log2-domain score of a = b = 1
    j = np.arange(n)
    b_j = torch.tensor(np.asarray(SCORE_PROFILES[profile](j, n), dtype=np.float64) / per_unit, dtype=torch.float32)
    a_i = 0.5 + torch.arange(L, dtype=torch.float32) / L
    a_i[::3] *= -1.0
    q = (a_i[:, None, None] * u[None] + 0.1 * torch.randn(L, H, D, generator=g)).to(torch.bfloat16).reshape(1, L, Cw)
    k_rows = (b_j[:, None, None] * u[None] + 0.1 * torch.randn(n, H, D, generator=g)).to(torch.bfloat16).reshape(n, Cw)
    v_rows = bf16_randn((n, Cw), 78)
    cap = (n + 127) // 128 * 128
    K, VT = pack_kv(k_rows, v_rows, H, cap)
    want = oracle.attention_dense(f64(q[0]).reshape(L, H, D), f64(k_rows).reshape(n, H, D),
                                  f64(v_rows).reshape(n, H, D)).reshape(L, Cw)
    o = torch.full((1, L, Cw), float("nan"), dtype=torch.bfloat16, device=DEV)
    binding.tuning_set("attn_splits", splits or None)
    binding.tuning_set("attn_waves", waves or None)
    try:
        ws = torch.empty(max(binding.attention_workspace_bytes(1, L, Cw, n), 256), dtype=torch.uint8, device=DEV)
        binding.attention_bf16(q.to(DEV), [K.to(DEV)], [VT.to(DEV)], [n], [cap], o, H, ws)
        torch.cuda.synchronize()
    finally:
        binding.tuning_set("attn_splits", None)
        binding.tuning_set("attn_waves", None)
    got = f64(o)
    assert np.isfinite(got).all()
    err = max_rel_err(got[0], want)
    assert err < 1e-2, err


def test_attention_full_size_480p_shape_sampled_queries():
    """Self-attention of the 14B 480p workload at steady state for one stream (4680 queries, 40 heads, 10 920 resident
    slots = 170 tiles and a tail of 40): whole output finite, 24 sampled queries x all heads against the oracle."""
    L, H, D, n = 4680, 40, 128, 10920
    Cw = H * D
    cap = (n + 63) // 64 * 64
    g = torch.Generator(device=DEV).manual_seed(11)
    q = torch.randn(1, L, Cw, generator=g, device=DEV).to(torch.bfloat16)
    k_rows = torch.randn(n, Cw, generator=g, device=DEV).to(torch.bfloat16)
    v_rows = torch.randn(n, Cw, generator=g, device=DEV).to(torch.bfloat16)
    K = torch.full((H, cap, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    VT = torch.full((H, D, cap), float("nan"), dtype=torch.bfloat16, device=DEV)
    K[:, :n, :] = k_rows.reshape(n, H, D).permute(1, 0, 2)
    VT[:, :, binding.vt_columns(cap)[:n].to(DEV)] = v_rows.reshape(n, H, D).permute(1, 2, 0)
    o = torch.full((1, L, Cw), float("nan"), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(max(binding.attention_workspace_bytes(1, L, Cw, n), 256), dtype=torch.uint8, device=DEV)
    binding.attention_bf16(q, [K], [VT], [n], [cap], o, H, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    rows = sorted(set(np.random.default_rng(1).integers(0, L, 20).tolist()) | {0, 127, 128, L - 1})
    want = oracle.attention_dense(f64(q[0, rows]).reshape(len(rows), H, D), f64(k_rows).reshape(n, H, D),
                                  f64(v_rows).reshape(n, H, D)).reshape(len(rows), Cw)
    assert max_rel_err(f64(o[0, rows]), want) < 1e-2


# ------------------------------------------------------------------------------------------ standalone cache
CACHE_CASES = [
    # P, S_frames, W_frames, heads, chunk sizes in frames (advance flag per chunk: True unless negative)
    (6, 1, 2, 1, [1, 1, 1, 1, 1, 1]),
    (15, 1, 6, 2, [3, 3, 3, 3, 3]),        # first chunk straddles sink and ring; third wraps mid-append
    (70, 0, 3, 1, [1, 2, 3, 1, 2]),        # no sink, tiles of 64 tokens with ragged tails
    (8, 2, 4, 3, [1, 1, 2, -2, 4, -4, 1]), # negative: same size again with advance = 0
]


@pytest.mark.parametrize("P,Sf,Wf,H,sizes", CACHE_CASES)
def test_append_evict_is_bit_exact(P, Sf, Wf, H, sizes):
    D = 128
    Cw = H * D
    S, W = Sf * P, Wf * P
    ccfg = binding.cache_cfg(2, 2, H, P, S, W)
    storage = torch.full((binding.kv_cache_bytes(ccfg),), 0xFF, dtype=torch.uint8, device=DEV)
    h = binding.kv_cache_init(ccfg, storage)
    layer, stream = 1, 1
    oc = oracle.RollingKVCache(S, W, P, Cw)
    for i, frames in enumerate(sizes):
        n = abs(frames) * P
        k = bf16_randn((n, Cw), 100 + i)
        v = bf16_randn((n, Cw), 200 + i)
        binding.kv_cache_append_evict(h, layer, stream, k.to(DEV), v.to(DEV), advance=frames > 0)
        oc.append_evict(f64(k), f64(v), advance=frames > 0)
        torch.cuda.synchronize()
        assert binding.kv_cache_state(h, layer, stream) == oc.state()
        want_map = oc.slot_map()
        assert binding.kv_cache_slot_map(h, layer, stream, S + W) == want_map.tolist()
        kp, vp, ip, cap = binding.kv_cache_device_ptrs(h, layer, stream)
        base = storage.data_ptr()
        nb = H * cap * D * 2
        K = storage[kp - base:kp - base + nb].view(torch.bfloat16).view(H, cap, D).permute(1, 0, 2).reshape(cap, Cw)
        V = storage[vp - base:vp - base + nb].view(torch.bfloat16).view(H, D, cap)
        V = V[:, :, binding.vt_columns(cap).to(DEV)].permute(2, 0, 1).reshape(cap, Cw)       # column order -> slot order
        ids = storage[ip - base:ip - base + cap * 8].view(torch.int64).cpu().numpy()
        live = want_map >= 0
        assert np.array_equal(ids[:S + W][live], want_map[live])
        ko, vo = oc.slot_contents()
        assert np.array_equal(f64(K)[:S + W][live], ko[live])          # copies: exact
        assert np.array_equal(f64(V)[:S + W][live], vo[live])
        # slots never written keep the poison
        assert torch.isnan(K[:S + W][torch.from_numpy(~live)].float()).all()
    # the other (layer, stream) pairs were not touched
    assert binding.kv_cache_state(h, 0, 0)["total"] == 0 and binding.kv_cache_state(h, 1, 0)["total"] == 0
    binding.kv_cache_reset(h, stream)
    assert binding.kv_cache_state(h, layer, stream)["total"] == 0
    binding.kv_cache_destroy(h)


def test_append_evict_errors_leave_state_untouched():
    P, H = 4, 1
    ccfg = binding.cache_cfg(1, 1, H, P, 4, 8)
    storage = torch.zeros(binding.kv_cache_bytes(ccfg), dtype=torch.uint8, device=DEV)
    h = binding.kv_cache_init(ccfg, storage)
    k = torch.zeros(4, 128, dtype=torch.bfloat16, device=DEV)
    binding.kv_cache_append_evict(h, 0, 0, k, k)
    before = binding.kv_cache_state(h, 0, 0)
    for bad_n, adv, code in ((12, True, binding.INVALID_ARG), (6, True, binding.INVALID_ARG), (8, False, binding.BAD_STATE)):
        kk = torch.zeros(bad_n, 128, dtype=torch.bfloat16, device=DEV)
        with pytest.raises(binding.Sdv2Error) as e:
            binding.kv_cache_append_evict(h, 0, 0, kk, kk, advance=adv)
        assert e.value.code == code
        assert binding.kv_cache_state(h, 0, 0) == before
    with pytest.raises(binding.Sdv2Error):
        binding.kv_cache_append_evict(h, 1, 0, k, k)
    binding.kv_cache_destroy(h)
