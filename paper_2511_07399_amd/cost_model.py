"""The paper's flop / byte model of causal-DiT inference (Appendix B) and the
algorithmic counts this build's benchmark prices its kernels with.

Host-side arithmetic only; nothing here touches the GPU.
"""

GIB = 1024 ** 3

# Appendix A: H100 SXM figures the paper's intensity uses.
H100_PEAK_FLOPS = 990e12
H100_REALISED_BW = 1.5e12

# MI355X published peaks used for this build's roofline fractions.
MI355X_BF16_FLOPS = 2.5e15
MI355X_HBM_BW = 8.0e12


def paper_flops(C, L_q, L_kv, N, b=1):
    """Appendix B, total compute: F = N (24 b L_q C^2 + 4 b L_q L_kv C)."""
    return N * (24 * b * L_q * C * C + 4 * b * L_q * L_kv * C)


def paper_bytes(C, L_q, L_kv, N, b=1, gamma=0.0):
    """Appendix B, memory movement: B = N (24 C^2 + 4 b L_kv C + 4 b L_q C + 36 b L_q C) + b gamma."""
    return N * (24 * C * C + 4 * b * L_kv * C + 4 * b * L_q * C + 36 * b * L_q * C) + b * gamma


def paper_intensity(C, L_q, L_kv, N, b=1, gamma=0.0, peak_flops=H100_PEAK_FLOPS, bandwidth=H100_REALISED_BW):
    """Appendix B, normalised hardware intensity: (F / peak) / (B / bandwidth); < 1 means memory-bound."""
    return (paper_flops(C, L_q, L_kv, N, b) / peak_flops) / (paper_bytes(C, L_q, L_kv, N, b, gamma) / bandwidth)


def gemm_flops(M, N, K):
    return 2 * M * N * K


def attention_flops(L_q, L_kv, C):
    """QK^T and PV over all heads: 4 L_q L_kv C (the Appendix B attention term for b = 1)."""
    return 4 * L_q * L_kv * C


def block_gemm_flops(rows, C, F):
    """QKV, out, cross q, cross out (C x C each, 6 C^2 in all) and the two FFN matrices."""
    return 2 * rows * (6 * C * C + 2 * C * F)


def block_flops(rows, C, F, L_kv, L_t):
    return block_gemm_flops(rows, C, F) + attention_flops(rows, L_kv, C) + attention_flops(rows, L_t, C)


def block_bytes(rows, C, F, L_kv, L_t):
    """Algorithmic bf16 bytes of one block: weights once, K/V read and written once, the
    paper's 36 bytes per token-channel of activation traffic, text K/V once."""
    weights = 2 * (6 * C * C + 2 * C * F)
    return weights + 4 * L_kv * C + 4 * rows * C + 36 * rows * C + 4 * L_t * C
