"""Pins of the latent I/O oracle (CPU only): patch embedding, output head, noise rate and sampler update.

None of these is printed in the paper (readings LIO1-LIO3 in oracle/latent_io.py); each is pinned against a library
routine (PyTorch's 3-D convolution and transposed convolution, layer_norm, linear) or a closed form of the
flow-matching interpolation, and the token count against Appendix B's 1 560 tokens per four-frame chunk at 480p.
"""

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2511_07399_amd import workloads as wk

T64 = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)


def rng(seed):
    return np.random.default_rng(seed)


def test_token_count_of_appendix_b():
    # 480 x 832 pixels, 8x VAE, 2 x 2 latent positions per token: 30 x 52 = 1 560 tokens per latent frame
    z = np.zeros((16, 1, 480 // 8, 832 // 8))
    assert oracle.patchify(z).shape == (1560, 64)
    assert wk.WORKLOADS["wan14b-480p-b4"].P == 1560


def test_patch_embedding_is_a_strided_3d_convolution():
    C, Fr, gh, gw = 24, 3, 4, 5
    z = rng(1).normal(size=(16, Fr, 2 * gh, 2 * gw))
    w, b = rng(2).normal(size=(C, 64)), rng(3).normal(size=C)
    got = oracle.patch_embed(z, w, b)
    conv = F.conv3d(T64(z)[None], T64(w).reshape(C, 16, 1, 2, 2), T64(b), stride=(1, 2, 2))[0]      # [C, F, gh, gw]
    want = conv.permute(1, 2, 3, 0).reshape(Fr * gh * gw, C).numpy()
    np.testing.assert_allclose(got, want, atol=1e-12)
    # token order: frame-major, then row, then column
    z2 = np.zeros_like(z)
    z2[:, 2, 2 * 3:2 * 3 + 2, 2 * 1:2 * 1 + 2] = 1.0
    hit = np.abs(oracle.patchify(z2)).sum(axis=1).nonzero()[0]
    assert hit.tolist() == [(2 * gh + 3) * gw + 1]


def test_unpatchify_is_the_inverse_and_a_transposed_convolution():
    Fr, gh, gw = 2, 3, 4
    tok = rng(4).normal(size=(Fr * gh * gw, 64))
    z = oracle.unpatchify(tok, Fr, gh, gw)
    np.testing.assert_array_equal(oracle.patchify(z), tok)
    t = T64(tok).reshape(Fr, gh, gw, 64).permute(3, 0, 1, 2)[None]                                 # [1, 64, F, gh, gw]
    want = F.conv_transpose3d(t, torch.eye(64, dtype=torch.float64).reshape(64, 16, 1, 2, 2), stride=(1, 2, 2))[0]
    np.testing.assert_allclose(z, want.numpy(), atol=1e-15)


def test_output_head_matches_torch():
    C, Fr, gh, gw = 32, 2, 3, 2
    L = Fr * gh * gw
    x = rng(5).normal(size=(L, C)) * 2 + 0.3
    tvec, table = rng(6).normal(size=C), rng(7).normal(size=(2, C))
    w, b = rng(8).normal(size=(64, C)), rng(9).normal(size=64)
    got = oracle.output_head(x, tvec, table, w, b, Fr, gh, gw)
    h = F.layer_norm(T64(x), (C,), eps=1e-6) * (1 + T64(table[1] + tvec)) + T64(table[0] + tvec)
    y = F.linear(h, T64(w), T64(b))                                                                  # [L, 64]
    t = y.reshape(Fr, gh, gw, 64).permute(3, 0, 1, 2)[None]
    want = F.conv_transpose3d(t, torch.eye(64, dtype=torch.float64).reshape(64, 16, 1, 2, 2), stride=(1, 2, 2))[0]
    np.testing.assert_allclose(got, want.numpy(), atol=1e-12)
    assert got.shape == (16, Fr, 2 * gh, 2 * gw)


def test_noise_rate_and_sampler_closed_forms():
    g = rng(10)
    x, e0, e1 = g.normal(size=(16, 1, 4, 4)), g.normal(size=(16, 1, 4, 4)), g.normal(size=(16, 1, 4, 4))
    np.testing.assert_array_equal(oracle.noise_latents(x, e0, 0.0), x)
    np.testing.assert_array_equal(oracle.noise_latents(x, e0, 1.0), e0)
    # with the exact velocity eps - x the clean estimate is x whatever the noise level, the last step returns it, and a
    # further step starts from the interpolation with the fresh noise
    for sigma in (0.9, 0.5, 0.05):
        z = oracle.noise_latents(x, e0, sigma)
        z_next, x0 = oracle.sampler_update(z, e0 - x, sigma, 0.0)
        np.testing.assert_allclose(x0, x, atol=1e-12)
        np.testing.assert_array_equal(z_next, x0)
        z_next, x0 = oracle.sampler_update(z, e0 - x, sigma, 0.3, e1)
        np.testing.assert_allclose(z_next, 0.7 * x + 0.3 * e1, atol=1e-12)
    # a chain of steps with an exact velocity model ends at x for any decreasing schedule
    sig = [0.8, 0.55, 0.3, 0.1, 0.0]
    eps = [g.normal(size=x.shape) for _ in sig]
    z = oracle.noise_latents(x, eps[0], sig[0])
    for i in range(len(sig) - 1):
        v = (z - x) / sig[i]                      # what an exact model returns at this point: eps_i - x
        z, _ = oracle.sampler_update(z, v, sig[i], sig[i + 1], eps[i + 1])
    np.testing.assert_allclose(z, x, atol=1e-10)
    # an error dv in the velocity moves the clean estimate by sigma dv, no more
    dv = g.normal(size=x.shape)
    _, x0 = oracle.sampler_update(oracle.noise_latents(x, e0, 0.4), e0 - x + dv, 0.4, 0.0)
    np.testing.assert_allclose(x0 - x, -0.4 * dv, atol=1e-12)


def test_latent_step_is_the_composition_and_moves_the_caches_once():
    wl = wk.WORKLOADS["tiny"]
    n_layers = 2
    layers = [wk.to_numpy(wk.block_weights(wl, layer)) for layer in range(n_layers)]
    mw, io = wk.to_numpy(wk.model_weights(wl)), wk.to_numpy(wk.io_weights(wl))
    ctx = wk.text_context(wl).double().numpy()
    text = [oracle.text_kv_prepare(ctx, w) for w in layers]
    mk = lambda: [oracle.RollingKVCache(wl.S, wl.W, wl.P, wl.C) for _ in range(n_layers)]
    ca, cb = mk(), mk()
    z = wk.latent_chunk(wl, 0).double().numpy()
    eps = wk.latent_chunk(wl, 0, kind=1).double().numpy()
    args = (mw, io, layers, ca, [t[0] for t in text], [t[1] for t in text], wl.H, wl.grid_h, wl.grid_w, 0)
    z1, x0 = oracle.denoise_latents_step(z, 0.7, 0.35, eps, *args)
    assert z1.shape == z.shape and ca[0].state()["total"] == wl.L
    x = oracle.patch_embed(z, io["W_pe"], io["b_pe"])
    x = oracle.denoise_step(x, mw, layers, cb, [t[0] for t in text], [t[1] for t in text], wl.H, wl.P, wl.grid_w, 0, t=700.0)
    v = oracle.output_head(x, oracle.timestep_vector(mw, 700.0), io["head_table"], io["W_head"], io["b_head"], 1, wl.grid_h, wl.grid_w)
    np.testing.assert_allclose(x0, z - 0.7 * v, atol=1e-12)
    np.testing.assert_allclose(z1, 0.65 * x0 + 0.35 * eps, atol=1e-12)
    # a second denoising step of the same chunk rewrites the cache in place
    oracle.denoise_latents_step(z1, 0.35, 0.0, None, *args, advance=False)
    assert ca[0].state()["total"] == wl.L
    # the timestep vector is the one the modulation is made from
    e0 = oracle.conditioning(mw, t=700.0)
    np.testing.assert_allclose(e0, oracle.conditioning(mw, tvec=oracle.timestep_vector(mw, 700.0)), atol=0)
