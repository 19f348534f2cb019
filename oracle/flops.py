"""Computation counts of Table 1 (scalar multiplications per layer per device)."""


def forward_mults_per_device(b, s, h, p):
    """(12 b s h^2 + 2 b s^2 h) / p."""
    return (12 * b * s * h * h + 2 * b * s * s * h) // p


def backward_mults_per_device(b, s, h, p, recompute=True):
    """Three forward passes' worth with activation checkpointing (one of them the
    recomputed forward), two without (Section 4)."""
    k = 3 if recompute else 2
    return k * forward_mults_per_device(b, s, h, p)


def gemm_flops_per_device(M, K, N, q):
    """One device's SUMMA product: 2 (M/q) K (N/q) flops."""
    return 2 * (M // q) * K * (N // q)
