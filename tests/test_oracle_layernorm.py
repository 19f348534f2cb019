"""Pins for oracle/layernorm.py: textbook two-pass definition, invariants,
2D partial statistics == 1D, finite differences for the backward formula."""
import numpy as np
import pytest

from oracle import layernorm as ln


def _rand(seed, M=6, h=16):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, h)) * 2.0 + 0.7
    gamma = 1.0 + 0.3 * rng.standard_normal(h)
    beta = 0.2 * rng.standard_normal(h)
    return rng, x, gamma, beta


def test_matches_two_pass_definition():
    _, x, gamma, beta = _rand(0)
    eps = 1e-5
    y, xhat, rstd = ln.forward(x, gamma, beta, eps)
    for r in range(x.shape[0]):           # python loops, population variance by its definition
        mu = sum(x[r]) / len(x[r])
        var = sum((v - mu) ** 2 for v in x[r]) / len(x[r])
        for c in range(x.shape[1]):
            want = (x[r, c] - mu) / np.sqrt(var + eps)
            assert abs(xhat[r, c] - want) < 1e-12
            assert abs(y[r, c] - (want * gamma[c] + beta[c])) < 1e-12
        assert abs(rstd[r] - 1 / np.sqrt(var + eps)) < 1e-12


def test_invariants():
    _, x, gamma, beta = _rand(1)
    eps = 1e-5
    _, xhat, rstd = ln.forward(x, gamma, beta, eps)
    var = x.var(axis=1)
    assert np.allclose(xhat.mean(axis=1), 0, atol=1e-13)                       # zero mean
    assert np.allclose(xhat.var(axis=1), var / (var + eps), atol=1e-12)        # unit variance up to eps
    y2, xhat2, _ = ln.forward(x + 5.0, gamma, beta, eps)                        # shift invariance
    assert np.allclose(xhat2, xhat, atol=1e-10)
    y0, xhat0, _ = ln.forward(x, np.ones_like(gamma), np.zeros_like(beta), eps)
    assert np.array_equal(y0, xhat0)


@pytest.mark.parametrize("q", [1, 2, 4])
def test_2d_partial_stats_equal_1d(q):
    _, x, gamma, beta = _rand(2, M=8, h=16)
    y, xhat, rstd = ln.forward(x, gamma, beta)
    r, c = 8 // q, 16 // q
    for i in range(q):
        for j in range(q):
            yb, xb, rs = ln.from_partial_stats(x, gamma, beta, q, i, j)
            assert np.allclose(yb, y[i * r:(i + 1) * r, j * c:(j + 1) * c], atol=1e-12)
            assert np.allclose(xb, xhat[i * r:(i + 1) * r, j * c:(j + 1) * c], atol=1e-12)
            assert np.allclose(rs, rstd[i * r:(i + 1) * r], atol=1e-12)
    st = ln.partial_stats(x, q, 0, 0)
    assert np.allclose(st[:, 0], x[:r, :c].sum(axis=1)) and np.allclose(st[:, 1], (x[:r, :c] ** 2).sum(axis=1))


def test_backward_finite_differences():
    rng, x, gamma, beta = _rand(3, M=3, h=8)
    dy = rng.standard_normal(x.shape)
    eps = 1e-5
    y, xhat, rstd = ln.forward(x, gamma, beta, eps)
    dx, dgamma, dbeta = ln.backward(dy, xhat, rstd, gamma)

    def loss(xx, gg, bb):
        return np.sum(dy * ln.forward(xx, gg, bb, eps)[0])

    hstep = 1e-6
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += hstep
        xm[idx] -= hstep
        assert abs((loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * hstep) - dx[idx]) < 1e-6
    for c in range(x.shape[1]):
        gp, gm = gamma.copy(), gamma.copy()
        gp[c] += hstep
        gm[c] -= hstep
        assert abs((loss(x, gp, beta) - loss(x, gm, beta)) / (2 * hstep) - dgamma[c]) < 1e-6
        bp, bm = beta.copy(), beta.copy()
        bp[c] += hstep
        bm[c] -= hstep
        assert abs((loss(x, gamma, bp) - loss(x, gamma, bm)) / (2 * hstep) - dbeta[c]) < 1e-6
    # orthogonality: each row of dx sums to 0 and is orthogonal to xhat
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-12)
    assert np.allclose((dx * xhat).sum(axis=1), 0, atol=1e-4)  # exact only as eps -> 0
