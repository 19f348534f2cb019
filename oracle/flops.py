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


def forward_operand_scalars(b, s, h):
    """Elements of the operands that enter the four forward SUMMA products of a layer (QKV, attention output,
    h -> 4h, 4h -> h): the quantity that Table 1's forward communication row multiplies by log(p) / (2 sqrt(p)),
    since every step of C = AB broadcasts one panel of A along rows and one of B along columns (Algorithm 1)."""
    M = b * s
    products = [(M, h, 3 * h), (M, h, h), (M, h, 4 * h), (M, 4 * h, h)]   # (rows of A, contraction, columns of B)
    return sum(m * k + k * n for (m, k, n) in products)
