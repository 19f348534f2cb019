"""Pins for oracle/summa.py and oracle/blocks.py (CPU only).

Nothing here compares the oracle with itself: brute-force Python loops,
closed forms, the Algorithm 1-3 virtual-grid replays, transpose identities and
finite differences of Eq. 1-3.
"""
import numpy as np
import pytest

from oracle import blocks, summa, flops
from oracle.metrics import rel_frobenius
from workloads import gemm_inputs, gemm_cases

FORMS = ["ab", "abt", "atb"]


def _shapes(form, M, K, N):
    return {"ab": ((M, K), (K, N)), "abt": ((M, K), (N, K)), "atb": ((K, M), (K, N))}[form]


@pytest.mark.parametrize("form", FORMS)
def test_brute_force_tiny(form):
    rng = np.random.default_rng(10)
    sa, sb = _shapes(form, 5, 7, 3)
    A, B = rng.standard_normal(sa), rng.standard_normal(sb)
    assert np.allclose(summa.product(form, A, B), summa.brute_matmul(form, A, B), rtol=0, atol=1e-13)


def test_brute_force_config1():
    # config 1's forward product itself (32 x 64 x 256), Python triple loop.
    g = [c for c in gemm_cases("config1") if c.form == "ab"][0]
    A, B = gemm_inputs(g.seed, g.form, g.M, g.K, g.N, g.dtype, g.dist_a, g.dist_b)
    want = summa.brute_matmul("ab", A, B)
    assert rel_frobenius(summa.matmul_ab(A, B), want) < 1e-14


@pytest.mark.parametrize("form", FORMS)
def test_not_symmetric_in_operands(form):
    # a transposed or swapped operand must be caught: use a rectangular, asymmetric case
    rng = np.random.default_rng(11)
    sa, sb = _shapes(form, 4, 6, 8)
    A, B = rng.standard_normal(sa), rng.standard_normal(sb)
    C = summa.product(form, A, B)
    assert C.shape == (4, 8)


def test_closed_forms():
    rng = np.random.default_rng(12)
    B = rng.standard_normal((6, 9))
    assert np.array_equal(summa.matmul_ab(np.eye(6), B), B)               # A = I
    assert np.array_equal(summa.matmul_ab(np.ones((4, 6)), np.ones((6, 9))), np.full((4, 9), 6.0))
    e = np.zeros((1, 6)); e[0, 2] = 1.0
    assert np.array_equal(summa.matmul_ab(e, B)[0], B[2])                 # one-hot row selects a row
    assert np.array_equal(summa.matmul_abt(e, B.T)[0], B[2])
    assert np.array_equal(summa.matmul_atb(e.T.copy(), B)[0], B[2])            # A[K,1] one-hot at k=2
    A = rng.standard_normal((6, 4))
    onehot = np.zeros((6, 1)); onehot[3, 0] = 1.0
    assert np.array_equal(summa.matmul_atb(A, onehot)[:, 0], A[3])        # A^T e_3 = row 3 of A


def test_transpose_identities():
    rng = np.random.default_rng(13)
    A, B = rng.standard_normal((5, 7)), rng.standard_normal((3, 7))
    assert np.allclose(summa.matmul_abt(A, B).T, summa.matmul_abt(B, A), atol=1e-14)   # (AB^T)^T = BA^T
    A2, B2 = rng.standard_normal((7, 5)), rng.standard_normal((7, 3))
    assert np.allclose(summa.matmul_atb(A2, B2).T, summa.matmul_atb(B2, A2), atol=1e-14)  # (A^T B)^T = B^T A
    assert np.allclose(summa.matmul_abt(A, B), summa.matmul_ab(A, B.T), atol=1e-14)
    assert np.allclose(summa.matmul_atb(A2, B2), summa.matmul_ab(A2.T, B2), atol=1e-14)


@pytest.mark.parametrize("q", [1, 2, 4])
@pytest.mark.parametrize("form", FORMS)
def test_reassembly_invariant(form, q):
    """Replaying Algorithms 1-3 on q*q virtual devices and reassembling the blocks
    gives the unpartitioned product; the owner-view index formulas give the same blocks."""
    rng = np.random.default_rng(14 + q)
    M, K, N = 8, 12, 16
    sa, sb = _shapes(form, M, K, N)
    A, B = rng.standard_normal(sa), rng.standard_normal(sb)
    Ab, Bb = blocks.partition(A, q), blocks.partition(B, q)
    Cb = {"ab": summa.grid_ab, "abt": summa.grid_abt, "atb": summa.grid_atb}[form](Ab, Bb)
    want = summa.brute_matmul(form, A, B)
    assert np.allclose(blocks.assemble(Cb), want, atol=1e-12)
    for i in range(q):
        for j in range(q):
            assert np.allclose(summa.owner_block(form, A, B, q, i, j), blocks.block(want, q, i, j), atol=1e-12)
            assert np.allclose(Cb[i, j], blocks.block(want, q, i, j), atol=1e-12)


def test_block_addressing_bit_exact():
    R, C, q = 6, 8, 2
    T = np.arange(R * C, dtype=np.int64).reshape(R, C)
    flat = blocks.pack_block_major(T, q)
    r, c = R // q, C // q
    # element (row, col) sits at ((i*q + j)*r + rr)*c + cc, by hand
    for row in range(R):
        for col in range(C):
            i, rr, j, cc = row // r, row % r, col // c, col % c
            assert flat[((i * q + j) * r + rr) * c + cc] == T[row, col]
    assert np.array_equal(blocks.unpack_block_major(flat, R, C, q), T)
    with pytest.raises(ValueError):
        blocks.partition(np.zeros((5, 8)), 2)


def _fd(f, X, dC, h=1e-6):
    """Central finite differences of <dC, f(X)> w.r.t. X."""
    G = np.zeros_like(X)
    for idx in np.ndindex(*X.shape):
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += h
        Xm[idx] -= h
        G[idx] = (np.sum(dC * f(Xp)) - np.sum(dC * f(Xm))) / (2 * h)
    return G


def test_differentiation_closure():
    """Eq. 1-3: each gradient is again one of the three products."""
    rng = np.random.default_rng(15)
    M, K, N = 3, 4, 5
    # Eq. 1: C = AB
    A, B, dC = rng.standard_normal((M, K)), rng.standard_normal((K, N)), rng.standard_normal((M, N))
    dA, dB = summa.grads_ab(A, B, dC)
    assert np.allclose(dA, _fd(lambda X: X @ B, A, dC), atol=1e-7)
    assert np.allclose(dB, _fd(lambda X: A @ X, B, dC), atol=1e-7)
    # Eq. 2: C = A^T B
    A, B = rng.standard_normal((K, M)), rng.standard_normal((K, N))
    dA, dB = summa.grads_atb(A, B, dC)
    assert np.allclose(dA, _fd(lambda X: X.T @ B, A, dC), atol=1e-7)
    assert np.allclose(dB, _fd(lambda X: A.T @ X, B, dC), atol=1e-7)
    # Eq. 3: C = A B^T
    A, B = rng.standard_normal((M, K)), rng.standard_normal((N, K))
    dA, dB = summa.grads_abt(A, B, dC)
    assert np.allclose(dA, _fd(lambda X: X @ B.T, A, dC), atol=1e-7)
    assert np.allclose(dB, _fd(lambda X: A @ X.T, B, dC), atol=1e-7)


def test_exact_integer_pattern_against_int64():
    # the pattern the GPU tests use: small integers => exact in any summation order
    M, K, N = 8, 16, 12
    A = ((np.arange(M)[:, None] * 3 + np.arange(K)[None, :] * 5) % 17 - 8).astype(np.int64)
    B = ((np.arange(K)[:, None] * 7 + np.arange(N)[None, :] * 2) % 13 - 6).astype(np.int64)
    assert np.array_equal(summa.matmul_ab(A, B).astype(np.int64), A @ B)
    assert np.array_equal(summa.matmul_abt(A, B.T.copy()).astype(np.int64), A @ B)
    assert np.array_equal(summa.matmul_atb(A.T.copy(), B).astype(np.int64), A @ B)


def test_flop_accounting_table1():
    """Table 1: forward multiplications per device = (12 b s h^2 + 2 b s^2 h)/p, from the per-op products."""
    b, s, h, n, q = 8, 1024, 4096, 32, 4
    p, M, d = q * q, b * s, h // n
    linear = sum(flops.gemm_flops_per_device(M, K, N, q) // 2
                 for (K, N) in [(h, 3 * h), (h, h), (h, 4 * h), (4 * h, h)])
    attn = (b // q) * (n // q) * (s * s * d + s * s * d)   # QK^T and PV, non-causal count
    assert linear + attn == flops.forward_mults_per_device(b, s, h, p)
    assert flops.backward_mults_per_device(b, s, h, p) == 3 * (linear + attn)
    assert flops.backward_mults_per_device(b, s, h, p, recompute=False) == 2 * (linear + attn)


def _table1():
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_costs.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, c1, c2 = line.split()
                rows[name] = (int(c1), int(c2))
    return rows


@pytest.mark.parametrize("b,s,h,p", [(8, 512, 1024, 16), (32, 512, 3072, 64), (8, 1024, 4096, 16), (4, 64, 128, 4)])
def test_counts_against_the_papers_table1(b, s, h, p):
    """The coefficients printed in Table 1 (fixture) against the oracle's counts, which are built from the shapes of
    the layer's products and not from these coefficients."""
    t = _table1()
    c1, c2 = t["forward_computation"]
    assert flops.forward_mults_per_device(b, s, h, p) == (c1 * b * s * h * h + c2 * b * s * s * h) // p
    c1, c2 = t["backward_computation"]
    assert flops.backward_mults_per_device(b, s, h, p) == (c1 * b * s * h * h + c2 * b * s * s * h) // p
    c1, c2 = t["forward_communication"]
    assert flops.forward_operand_scalars(b, s, h) == c1 * b * s * h + c2 * h * h
    c1, c2 = t["backward_communication"]
    assert 3 * flops.forward_operand_scalars(b, s, h) == c1 * b * s * h + c2 * h * h
