"""Oracle of the steps between latents and the blocks' hidden state (TEST INFRASTRUCTURE ONLY).

The paper runs a causal DiT "built on Wan 2.1 and CausVid" on VAE latents in 1-4 denoising steps
per chunk (Section 5.1), at 1 560 tokens for a chunk of four video frames at 480p (Appendix B:
480 x 832 pixels -> 60 x 104 latent positions -> 30 x 52 tokens, i.e. 2 x 2 latent positions per
token), and sets a per-chunk NOISE RATE s_t for the incoming frames (Section 4.1, motion-aware
noise scheduler).  It prints none of: the patch embedding, the output head, the update between
denoising steps.  Everything below is therefore this build's reading ("parity unpinned" against
the paper), written as the plain definitions and pinned against library routines and closed forms:

  LIO1  patch embedding: a latent chunk z [16, F, 2 gh, 2 gw] becomes F gh gw tokens, token (f, r, c)
        holding the 64 numbers z[ch, f, 2r + dr, 2c + dc] in the order (ch, dr, dc); x = patch W_pe^T + b_pe.
        This is a 3-D convolution with kernel and stride (1, 2, 2).
  LIO2  output head: y = (LN(x) (1 + scale) + shift) W_head^T + b_head with (shift, scale) =
        head_table[2, C] + tvec, 64 numbers per token laid back into [16, F, 2 gh, 2 gw] in the same order.
  LIO3  noise rate and sampler (flow-matching form): a clean latent x and noise eps at rate s give
        (1 - s) x + s eps; the blocks' output is read as the velocity v = eps - x, so at noise level
        sigma the clean estimate is x0 = z - sigma v; a further denoising step starts from
        (1 - sigma') x0 + sigma' eps' with fresh noise eps' (passed in), the last one returns x0.
        The timestep fed to the blocks is 1000 sigma.
"""

import numpy as np

from .dit_block import denoise_step, layer_norm, linear, timestep_vector

LATENT_CHANNELS = 16


def patchify(z):
    """z [Cl, F, Hl, Wl] -> tokens [F (Hl/2) (Wl/2), 4 Cl]; tokens frame-major then row then column."""
    Cl, F, Hl, Wl = z.shape
    gh, gw = Hl // 2, Wl // 2
    out = np.empty((F * gh * gw, Cl * 4), dtype=z.dtype)
    for f in range(F):
        for r in range(gh):
            for c in range(gw):
                out[(f * gh + r) * gw + c] = z[:, f, 2 * r:2 * r + 2, 2 * c:2 * c + 2].reshape(-1)
    return out


def unpatchify(tok, F, gh, gw):
    """The inverse of patchify: tokens [F gh gw, 4 Cl] -> [Cl, F, 2 gh, 2 gw]."""
    Cl = tok.shape[1] // 4
    z = np.empty((Cl, F, 2 * gh, 2 * gw), dtype=tok.dtype)
    for f in range(F):
        for r in range(gh):
            for c in range(gw):
                z[:, f, 2 * r:2 * r + 2, 2 * c:2 * c + 2] = tok[(f * gh + r) * gw + c].reshape(Cl, 2, 2)
    return z


def patch_embed(z, w_pe, b_pe, dtype=np.float64):
    """Hidden state [L, C] of a latent chunk: x = patchify(z) W_pe^T + b_pe, W_pe [C, 64]."""
    f = lambda a: np.asarray(a, dtype=dtype)
    return linear(patchify(f(z)), f(w_pe), f(b_pe))


def output_head(x, tvec, head_table, w_head, b_head, F, gh, gw, dtype=np.float64):
    """[L, C] -> [16, F, 2 gh, 2 gw]: modulated LayerNorm, projection to 64 numbers per token, un-patching."""
    f = lambda a: np.asarray(a, dtype=dtype)
    mod = f(head_table) + f(tvec)[None, :]
    h = layer_norm(f(x)) * (1.0 + mod[1]) + mod[0]
    return unpatchify(linear(h, f(w_head), f(b_head)), F, gh, gw)


def noise_latents(x, eps, s):
    """A clean latent at noise rate s: (1 - s) x + s eps."""
    return (1.0 - s) * x + s * eps


def sampler_update(z, v, sigma, sigma_next, eps_next=None):
    """One update of the few-step sampler: x0 = z - sigma v; the next step's input (1 - sigma') x0 + sigma' eps',
    or x0 itself when sigma' = 0.  Returns (z_next, x0)."""
    x0 = z - sigma * v
    if sigma_next == 0.0:
        return x0, x0
    return noise_latents(x0, eps_next, sigma_next), x0


def denoise_latents_step(z, sigma, sigma_next, eps_next, mw, io, block_ws, caches, text_ks, text_vs, n_heads, grid_h,
                         grid_w, frame_pos0, advance=True, dtype=np.float64):
    """Latents in, latents out: patch embedding, the N blocks at timestep 1000 sigma, output head, sampler update.
    z [16, F, 2 grid_h, 2 grid_w].  Returns (z_next, x0)."""
    F = z.shape[1]
    t = 1000.0 * sigma
    x = patch_embed(z, io["W_pe"], io["b_pe"], dtype)
    x = denoise_step(x, mw, block_ws, caches, text_ks, text_vs, n_heads, grid_h * grid_w, grid_w, frame_pos0,
                     advance=advance, t=t, dtype=dtype)
    v = output_head(x, timestep_vector(mw, t, dtype), io["head_table"], io["W_head"], io["b_head"], F, grid_h, grid_w,
                    dtype)
    return sampler_update(np.asarray(z, dtype=dtype), v, sigma, sigma_next, eps_next)
