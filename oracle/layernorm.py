"""Layer normalisation over the hidden dimension (Section 3.2.2).

xhat = (x - E[x]) / sqrt(Var[x] + eps) with E[x] = (1/h) sum x and
Var[x] = E[x^2] - E[x]^2, followed by the affine map y = gamma * xhat + beta.
The 2D form computes sum x and sum x^2 per device block and adds the q
partials of a grid row; ``partial_stats`` / ``from_partial_stats`` spell that
out so that it can be compared with the unpartitioned definition.
"""
import numpy as np

from . import blocks as _b

EPS_DEFAULT = 1e-5


def forward(x, gamma, beta, eps=EPS_DEFAULT):
    """Returns y, xhat, rstd (rstd = 1/sqrt(Var+eps), one per row)."""
    x = np.asarray(x, dtype=np.float64)
    h = x.shape[1]
    mean = x.sum(axis=1) / h
    meansq = (x * x).sum(axis=1) / h
    var = meansq - mean * mean
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mean[:, None]) * rstd[:, None]
    y = xhat * np.asarray(gamma, dtype=np.float64)[None, :] + np.asarray(beta, dtype=np.float64)[None, :]
    return y, xhat, rstd


def backward(dy, xhat, rstd, gamma):
    """Gradient of the input given dJ/dy, plus dgamma and dbeta.

    With g = dJ/dxhat = dy * gamma:
    dx = rstd * ( g - xhat * (1/h) sum_j xhat_j g_j - (1/h) sum_j g_j ).
    """
    dy = np.asarray(dy, dtype=np.float64)
    xhat = np.asarray(xhat, dtype=np.float64)
    rstd = np.asarray(rstd, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    h = dy.shape[1]
    g = dy * gamma[None, :]
    s_xg = (xhat * g).sum(axis=1) / h
    s_g = g.sum(axis=1) / h
    dx = rstd[:, None] * (g - xhat * s_xg[:, None] - s_g[:, None])
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    return dx, dgamma, dbeta


# ---- the 2D decomposition ---------------------------------------------------
def partial_stats(x, q, i, l):
    """What device (i, l) contributes to the row all-reduce: [M/q, 2] = (sum x, sum x^2)."""
    blk = np.asarray(_b.block(x, q, i, l), dtype=np.float64)
    return np.stack([blk.sum(axis=1), (blk * blk).sum(axis=1)], axis=1)


def from_partial_stats(x, gamma, beta, q, i, j, eps=EPS_DEFAULT):
    """Device (i, j)'s output block computed the 2D way: add q partials, normalise own block."""
    h = x.shape[1]
    tot = sum(partial_stats(x, q, i, l) for l in range(q))
    mean = tot[:, 0] / h
    var = tot[:, 1] / h - mean * mean
    rstd = 1.0 / np.sqrt(var + eps)
    blk = np.asarray(_b.block(x, q, i, j), dtype=np.float64)
    xhat = (blk - mean[:, None]) * rstd[:, None]
    g = np.asarray(_b.vector_slice(np.asarray(gamma), q, j), dtype=np.float64)
    b = np.asarray(_b.vector_slice(np.asarray(beta), q, j), dtype=np.float64)
    return xhat * g[None, :] + b[None, :], xhat, rstd
