"""Pins for oracle/model_ends.py: the embedding as the one-hot product of the paper (also replayed as Algorithm 1
on a virtual grid), its gradient as the transposed one-hot product, cross entropy by brute force, closed forms,
scipy's logsumexp and finite differences (which also settle the garbled soft-max formula)."""
import math

import numpy as np

from oracle import blocks, model_ends as me, summa
from workloads import token_inputs


def test_embedding_is_the_one_hot_product_and_summa_replay():
    rng = np.random.default_rng(0)
    b, s, v, h, q = 4, 6, 16, 8, 2
    tokens, _ = token_inputs(1, b, s, v)
    table = rng.standard_normal((v, h))
    X = me.embedding(tokens, table)
    assert X.shape == (b * s, h)
    for t in range(b * s):
        assert np.array_equal(X[t], table[tokens[t]])
    assert np.array_equal(X, me.one_hot(tokens, v) @ table)
    # Algorithm 1 on the one-hot matrix partitioned q x q: the 2D form the paper describes
    Xb = summa.grid_ab(blocks.partition(me.one_hot(tokens, v), q), blocks.partition(table, q))
    assert np.array_equal(blocks.assemble(Xb), X)


def test_embedding_grad_is_transposed_product_and_derivative():
    rng = np.random.default_rng(1)
    b, s, v, h = 3, 5, 7, 4
    tokens, _ = token_inputs(2, b, s, v)
    d_x = rng.standard_normal((b * s, h))
    G = me.embedding_grad(tokens, d_x, v)
    assert np.allclose(G, me.one_hot(tokens, v).T @ d_x, atol=1e-14)
    absent = np.setdiff1d(np.arange(v), tokens)
    assert np.all(G[absent] == 0.0)
    # <d_x, embedding(table)> is linear in the table with derivative G
    table = rng.standard_normal((v, h))
    E = np.zeros_like(table)
    E[tokens[0], 2] = 1.0
    assert abs(np.sum(d_x * me.embedding(tokens, table + E)) - np.sum(d_x * me.embedding(tokens, table)) - G[tokens[0], 2]) < 1e-12


def test_lm_head_is_abt():
    rng = np.random.default_rng(2)
    Hd, T = rng.standard_normal((6, 4)), rng.standard_normal((9, 4))
    assert np.array_equal(me.lm_head(Hd, T), summa.matmul_abt(Hd, T))
    assert np.allclose(me.lm_head(Hd, T)[2, 5], sum(Hd[2, e] * T[5, e] for e in range(4)), atol=1e-14)


def test_cross_entropy_brute_force_closed_forms_and_library():
    from scipy.special import logsumexp
    rng = np.random.default_rng(3)
    n, v = 5, 11
    x = rng.standard_normal((n, v)) * 3
    labels = rng.integers(0, v, n)
    H, L = me.cross_entropy(x, labels)
    for t in range(n):
        Z = sum(math.exp(x[t, i]) for i in range(v))
        assert abs(H[t] - (math.log(Z) - x[t, labels[t]])) < 1e-12
        assert abs(H[t] + math.log(math.exp(x[t, labels[t]]) / Z)) < 1e-12      # H = -log q_l
    assert np.allclose(L, logsumexp(x, axis=1), atol=1e-13)
    H0, _ = me.cross_entropy(np.zeros((n, v)), labels)
    assert np.allclose(H0, math.log(v), atol=1e-14)                              # uniform prediction
    big = np.zeros((n, v)); big[np.arange(n), labels] = 50.0
    assert np.all(me.cross_entropy(big, labels)[0] < 1e-20 * 1e3)                # certain and right: loss ~ 0
    shifted, _ = me.cross_entropy(x + 7.0, labels)
    assert np.allclose(shifted, H, atol=1e-12)                                   # invariant to a row shift
    huge, _ = me.cross_entropy(x + 1e4, labels)
    assert np.all(np.isfinite(huge)) and np.allclose(huge, H, atol=1e-8)          # no overflow


def test_cross_entropy_grad_finite_differences_and_row_sums():
    rng = np.random.default_rng(4)
    n, v = 4, 6
    x = rng.standard_normal((n, v))
    labels = rng.integers(0, v, n)
    G = me.cross_entropy_grad(x, labels, scale=0.25)
    assert np.allclose(G.sum(axis=1), 0.0, atol=1e-14)          # q sums to one, minus the one-hot
    hstep = 1e-6
    for idx in np.ndindex(n, v):
        p, m = x.copy(), x.copy()
        p[idx] += hstep
        m[idx] -= hstep
        fd = 0.25 * (me.cross_entropy(p, labels)[0].sum() - me.cross_entropy(m, labels)[0].sum()) / (2 * hstep)
        assert abs(fd - G[idx]) < 1e-8, idx
    # the formula as printed (q_j = x_j / sum exp) does not have this derivative: the exponential belongs there
    q_printed = x / np.exp(x).sum(axis=1, keepdims=True)
    q_printed[np.arange(n), labels] -= 1.0
    assert not np.allclose(0.25 * q_printed, G, atol=1e-3)


def test_token_generator_shape_and_skew():
    tokens, labels = token_inputs(5, 8, 64, 1000)
    assert tokens.dtype == np.int32 and tokens.shape == (512,) and labels.shape == (512,)
    assert tokens.min() >= 0 and tokens.max() < 1000
    assert np.mean(tokens < 10) > 0.25                      # Zipf: the ten most frequent indices carry > 1/4 of the mass
    t2, _ = token_inputs(5, 8, 64, 1000)
    assert np.array_equal(tokens, t2)
