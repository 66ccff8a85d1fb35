"""GPU parity of the steps between latents and the blocks' hidden state (sdv2_patch_embed, sdv2_output_head,
sdv2_noise_latents, sdv2_sampler_update, sdv2_timestep_vector, sdv2_denoise_latents_step) against oracle/latent_io.py.

Bars (max |gpu - oracle| / max |oracle|): the patch embedding and the two elementwise updates take bf16-exact inputs
and accumulate in fp32, so they hold 1e-5; everything that passes through a bf16 activation (the head's LayerNorm
output, the blocks) holds the block tests' 2e-2.  The sampler's result is also compared on the update alone
(z - x0 = sigma v), since z_next itself is dominated by z.
"""

import numpy as np
import pytest
import torch

import oracle
from paper_2511_07399_amd import binding, workloads as wk
from parity_util import GpuRunner, OracleRunner, max_rel_err, visible_branches

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_EXACT = 1e-5
TOL_X = 2e-2


def cfg_of(wl, n_layers=1):
    binding.load_library()
    return binding.model_cfg(wl.C, wl.H, wl.F, wl.grid_h, wl.grid_w, wl.L_t, n_layers, wl.t_dim)


def io_of(wl):
    host = wk.io_weights(wl)
    dev = {k: v.to(DEV) for k, v in host.items()}
    return wk.to_numpy(host), dev, binding.io_weights(dev)


@pytest.mark.parametrize("name,B", [("tiny", 1), ("tiny", 3), ("wan1.3b-block", 2), ("wan14b-480p-b4", 2)])
def test_patch_embed(name, B):
    wl = wk.WORKLOADS[name]
    cfg = cfg_of(wl)
    io_np, io_dev, io = io_of(wl)
    z = torch.stack([wk.latent_chunk(wl, 0, s) for s in range(B)])
    x = torch.full((B, wl.L, wl.C), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(binding.latent_io_workspace_bytes(cfg, B, wl.L), dtype=torch.uint8, device=DEV)
    binding.patch_embed(cfg, io, z.to(DEV).contiguous(), x, ws)
    torch.cuda.synchronize()
    for s in range(B):
        want = oracle.patch_embed(z[s].double().numpy(), io_np["W_pe"], io_np["b_pe"])
        assert max_rel_err(x[s].cpu().numpy(), want) < TOL_EXACT, (name, s)


@pytest.mark.parametrize("name,B", [("tiny", 1), ("tiny", 3), ("wan1.3b-block", 2), ("wan14b-480p-b4", 2)])
def test_output_head(name, B):
    wl = wk.WORKLOADS[name]
    cfg = cfg_of(wl)
    io_np, io_dev, io = io_of(wl)
    # rows with a mean and a spread of their own, so that the LayerNorm has something to remove
    x = torch.stack([wk.chunk_input(wl, 1, s) * (1.0 + 0.5 * s) + 0.25 * (s + 1) for s in range(B)])
    tvec = torch.stack([wk.timestep_vector(wl, 1, 0, s) for s in range(B)])
    v = torch.full((B, wk.LATENT_CHANNELS, wl.frames_per_chunk, 2 * wl.grid_h, 2 * wl.grid_w), float("nan"),
                   dtype=torch.float32, device=DEV)
    ws = torch.empty(binding.latent_io_workspace_bytes(cfg, B, wl.L), dtype=torch.uint8, device=DEV)
    binding.output_head(cfg, io, x.to(DEV).contiguous(), tvec.to(DEV).contiguous(), v, ws)
    torch.cuda.synchronize()
    for s in range(B):
        want = oracle.output_head(x[s].double().numpy(), tvec[s].double().numpy(), io_np["head_table"], io_np["W_head"],
                                  io_np["b_head"], wl.frames_per_chunk, wl.grid_h, wl.grid_w)
        assert max_rel_err(v[s].cpu().numpy(), want) < TOL_X, (name, s)


def test_noise_and_sampler_update():
    wl = wk.WORKLOADS["wan1.3b-block"]
    B = 3
    z = torch.stack([wk.latent_chunk(wl, 2, s) for s in range(B)])
    v = torch.stack([wk.latent_chunk(wl, 2, s, kind=1) for s in range(B)])
    eps = torch.stack([wk.latent_chunk(wl, 2, s, kind=2) for s in range(B)])
    zd, vd, ed = (t.to(DEV).contiguous() for t in (z, v, eps))
    rates = [0.0, 0.625, 1.0]
    out = torch.empty_like(zd)
    binding.noise_latents(zd, ed, out, rates)
    sig, sig_next = [1.0, 0.75, 0.5], [0.5, 0.0, 0.5]
    z_next, x0 = torch.empty_like(zd), torch.empty_like(zd)
    binding.sampler_update(zd, vd, ed, z_next, x0, sig, sig_next)
    in_place = zd.clone()
    binding.sampler_update(in_place, vd, ed, in_place, None, sig, sig_next)
    torch.cuda.synchronize()
    for s in range(B):
        f = lambda t: t[s].double().numpy()
        assert max_rel_err(out[s].cpu().numpy(), oracle.noise_latents(f(z), f(eps), rates[s])) < TOL_EXACT
        want_next, want_x0 = oracle.sampler_update(f(z), f(v), sig[s], sig_next[s], f(eps))
        assert max_rel_err(z_next[s].cpu().numpy(), want_next) < TOL_EXACT
        assert max_rel_err(x0[s].cpu().numpy(), want_x0) < TOL_EXACT
    assert torch.equal(in_place, z_next)
    # rate 0 and 1 return the operands themselves; sigma_next = 0 returns x0
    assert torch.equal(out[0], zd[0]) and torch.equal(out[2], ed[2])
    assert torch.equal(z_next[1], x0[1])


def test_sampler_update_without_noise_when_last_step():
    wl = wk.WORKLOADS["tiny"]
    z = wk.latent_chunk(wl, 0).unsqueeze(0).to(DEV).contiguous()
    v = wk.latent_chunk(wl, 0, kind=1).unsqueeze(0).to(DEV).contiguous()
    z_next = torch.empty_like(z)
    binding.sampler_update(z, v, None, z_next, None, [0.5], [0.0])
    torch.cuda.synchronize()
    want, _ = oracle.sampler_update(z[0].cpu().double().numpy(), v[0].cpu().double().numpy(), 0.5, 0.0)
    assert max_rel_err(z_next[0].cpu().numpy(), want) < TOL_EXACT
    with pytest.raises(binding.Sdv2Error):
        binding.sampler_update(z, v, None, z_next, None, [0.5], [0.25])        # a further step needs its noise
    with pytest.raises(binding.Sdv2Error):
        binding.sampler_update(z, v, v, z_next, None, [0.5], [0.75])           # sigma must not grow
    with pytest.raises(binding.Sdv2Error):
        binding.noise_latents(z, v, z_next, [1.5])


@pytest.mark.parametrize("name", ["tiny", "wan1.3b-block"])
def test_timestep_vector(name):
    wl = wk.WORKLOADS[name]
    gpu = GpuRunner(wl, n_layers=1, n_streams=1)
    mw_np = wk.to_numpy(wk.model_weights(wl))
    ts = [0.0, 250.0, 999.0]
    tvec = torch.empty(len(ts), wl.C, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(binding.conditioning_workspace_bytes(gpu.cfg, len(ts)), 256), dtype=torch.uint8, device=DEV)
    binding.timestep_vector(gpu.cfg, gpu.mw, ts, tvec, ws)
    torch.cuda.synchronize()
    for i, t in enumerate(ts):
        assert max_rel_err(tvec[i].cpu().numpy(), oracle.timestep_vector(mw_np, t)) < 2e-3, (name, t)
    gpu.close()


def run_latents_both(wl, n_layers, n_chunks, sigmas, edit=None, n_streams=1):
    """n_chunks chunks per stream, each taken through the noise levels ``sigmas`` (ending at 0), B = n_streams rows
    per call.  Returns the errors of z after every step, of the update of every step, and whether the cache state
    matches after every chunk."""
    gpu = GpuRunner(wl, n_layers=n_layers, n_streams=n_streams, edit=edit)
    ora = OracleRunner(wl, n_layers=n_layers, n_streams=n_streams, edit=edit)
    io_np = wk.to_numpy(wk.io_weights(wl))
    gpu.io()
    levels = list(sigmas) + [0.0]
    res = {"z": [], "upd": [], "state_equal": True}
    for chunk in range(n_chunks):
        clean = [wk.latent_chunk(wl, chunk, s) for s in range(n_streams)]
        eps0 = [wk.latent_chunk(wl, chunk, s, kind=1) for s in range(n_streams)]
        zo = [oracle.noise_latents(clean[s].double().numpy(), eps0[s].double().numpy(), levels[0]) for s in range(n_streams)]
        zg = torch.empty(n_streams, *clean[0].shape, dtype=torch.float32, device=DEV)
        binding.noise_latents(torch.stack(clean).to(DEV).contiguous(), torch.stack(eps0).to(DEV).contiguous(), zg,
                              [levels[0]] * n_streams)
        x0g = torch.empty_like(zg)
        for step in range(len(sigmas)):
            sg, sn = levels[step], levels[step + 1]
            eps = [wk.latent_chunk(wl, chunk, s, kind=2 + step) for s in range(n_streams)]
            descs = [(s, chunk * wl.frames_per_chunk, wl.frames_per_chunk, 1 if step == 0 else 0) for s in range(n_streams)]
            before = zg.clone()
            gpu.denoise_latents(zg, descs, [sg] * n_streams, [sn] * n_streams,
                                eps_next=torch.stack(eps).to(DEV).contiguous() if sn > 0 else None, x0=x0g)
            torch.cuda.synchronize()
            for s in range(n_streams):
                z_in = zo[s]
                zo[s], x0 = oracle.denoise_latents_step(
                    z_in, sg, sn, eps[s].double().numpy(), ora.mw, io_np, [ora.layers[l] for l in range(n_layers)],
                    [ora.caches[l][s] for l in range(n_layers)], [ora.text[l][s][0] for l in range(n_layers)],
                    [ora.text[l][s][1] for l in range(n_layers)], wl.H, wl.grid_h, wl.grid_w,
                    chunk * wl.frames_per_chunk, advance=step == 0)
                res["z"].append(max_rel_err(zg[s].cpu().numpy(), zo[s]))
                res["upd"].append(max_rel_err((before[s] - x0g[s]).cpu().numpy(), z_in - x0))
                # the next step starts from the oracle's own latents on both sides, so that each step is judged alone
                zg[s].copy_(torch.from_numpy(zo[s]).float())
                zo[s] = zg[s].cpu().double().numpy()
        for layer in range(n_layers):
            for s in range(n_streams):
                res["state_equal"] &= gpu.state(layer, s) == ora.caches[layer][s].state()
    gpu.close()
    return res


def test_denoise_latents_step_tiny_two_steps_through_eviction():
    wl = wk.WORKLOADS["tiny"]
    res = run_latents_both(wl, n_layers=2, n_chunks=5, sigmas=(1.0, 0.5), edit=visible_branches(wl))
    assert res["state_equal"]
    assert max(res["z"]) < TOL_X, res["z"]
    assert max(res["upd"]) < TOL_X, res["upd"]


def test_denoise_latents_step_tiny_batched_four_steps():
    wl = wk.WORKLOADS["tiny"]
    res = run_latents_both(wl, n_layers=2, n_chunks=2, sigmas=(1.0, 0.75, 0.5, 0.25), edit=visible_branches(wl),
                           n_streams=3)
    assert res["state_equal"]
    assert max(res["upd"]) < TOL_X, res["upd"]
    assert max(res["z"]) < TOL_X, res["z"]


def test_denoise_latents_step_1p3b_two_layers():
    wl = wk.WORKLOADS["wan1.3b-block"]
    res = run_latents_both(wl, n_layers=2, n_chunks=2, sigmas=(0.8, 0.4), edit=visible_branches(wl))
    assert res["state_equal"]
    assert max(res["upd"]) < TOL_X, res["upd"]
    assert max(res["z"]) < TOL_X, res["z"]


def test_denoise_latents_step_refusals_leave_the_cache_alone():
    wl = wk.WORKLOADS["tiny"]
    gpu = GpuRunner(wl, n_layers=1, n_streams=1)
    z = wk.latent_chunk(wl, 0).unsqueeze(0).to(DEV).contiguous()
    keep = z.clone()
    desc = [(0, 0, wl.frames_per_chunk, 1)]
    before = gpu.state(0, 0)
    with pytest.raises(binding.Sdv2Error):
        gpu.denoise_latents(z, desc, [0.5], [0.75])                     # sigma grows
    with pytest.raises(binding.Sdv2Error):
        gpu.denoise_latents(z, desc, [0.0], [0.0])                      # nothing to denoise at sigma = 0
    with pytest.raises(binding.Sdv2Error):
        gpu.denoise_latents(z, desc, [0.5], [0.25])                     # eps_next missing
    with pytest.raises(binding.Sdv2Error):
        gpu.denoise_latents(z, [(5, 0, wl.frames_per_chunk, 1)], [0.5], [0.0])     # no such stream
    torch.cuda.synchronize()
    assert gpu.state(0, 0) == before
    assert torch.equal(z, keep)
    gpu.close()
