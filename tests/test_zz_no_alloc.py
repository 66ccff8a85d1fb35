"""sdv2_gemm_bf16_noalloc (the entry point that allocates nothing) against sdv2_gemm_bf16 with a caller workspace.

Two calls in a row share the library's built-in scratch array; the second is smaller and lays its partial sums out
differently, so stale contents of the first would show.  Bar: the two entry points run the same kernels on the same
plan, so their outputs are equal bit for bit; both are also held to the per-kernel bar against the oracle.
"""

import numpy as np
import pytest
import torch

from oracle.dit_block import linear as oracle_linear
from paper_2511_07399_amd import binding
from parity_util import max_rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(torch.bfloat16)


def one_case(M, N, K, epi, seed):
    a, w = draw((M, K), seed).to(DEV), draw((N, K), seed + 1, 0.05).to(DEV)
    bias = draw((N,), seed + 2, 0.5).float().to(DEV)
    gate_a = draw((N,), seed + 3, 0.3).float().to(DEV)
    gate_b = draw((1, N), seed + 4, 0.3).float().to(DEV)
    x0 = draw((M, N), seed + 5).float().to(DEV)
    ws_bytes = binding.gemm_workspace_bytes(M, N, K, epi)
    assert 0 < ws_bytes <= binding.gemm_noalloc_max_scratch_bytes(), "the case must split k and fit the scratch"
    ws = torch.full((ws_bytes // 4,), float("nan"), dtype=torch.float32, device=DEV)
    want_out = x0.clone() if epi >= 2 else torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    binding.gemm_bf16(a, w, bias, want_out, epi, gate_a, gate_b, N, M, workspace=ws)
    got_out = x0.clone() if epi >= 2 else torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    binding.gemm_bf16_noalloc(a, w, bias, got_out, epi, gate_a, gate_b, N, M)
    torch.cuda.synchronize()
    assert torch.equal(got_out, want_out), "no-alloc entry point differs from the workspace entry point"
    acc = oracle_linear(a.cpu().double().numpy(), w.cpu().double().numpy(), bias.cpu().double().numpy())
    if epi == 2:
        gate = (gate_a + gate_b[0]).cpu().double().numpy()
        ref = x0.cpu().double().numpy() + gate[None, :] * acc
    else:
        ref = acc
    assert max_rel_err(got_out.cpu().double().numpy(), ref) < (1e-4 if epi >= 2 else 1e-2)


def test_noalloc_gemm_two_calls_in_a_row_second_smaller():
    # FFN-2 of the 1.3B block with two streams (two k parts of 2048 rows), then with one (four parts of 1024 rows)
    one_case(2048, 1536, 8960, 2, 100)
    one_case(1024, 1536, 8960, 2, 200)
    # a forced split on a small ragged shape, bf16 output
    binding.tuning_set("gemm_tile", "1,4,2,2")
    try:
        one_case(300, 512, 1024, 0, 300)
    finally:
        binding.tuning_set("gemm_tile", None)


def test_noalloc_gemm_rejects_what_does_not_fit():
    # FFN-2 of the 14B block splits k in three parts of 1024 x 5120 floats: 63 MB
    M, N, K = 1024, 5120, 13824
    assert binding.gemm_workspace_bytes(M, N, K, 2) > binding.gemm_noalloc_max_scratch_bytes()
    a, w = torch.zeros(M, K, dtype=torch.bfloat16, device=DEV), torch.zeros(N, K, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(M, N, dtype=torch.float32, device=DEV)
    g = torch.zeros(N, dtype=torch.float32, device=DEV)
    with pytest.raises(binding.Sdv2Error) as e:
        binding.gemm_bf16_noalloc(a, w, None, out, 2, g, g.reshape(1, N), N, M)
    assert e.value.code == binding.INVALID_ARG
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
