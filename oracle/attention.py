"""Multi-head self-attention on whole sequences (Sections 2.1 and 3.2.1).

For one sequence and one head with Q, K, V of shape [s, d]:
S = Q K^T / sqrt(d), optional causal mask (-inf strictly above the diagonal),
P = row softmax(S), O = P V.  In the 2D scheme a device holds n/q heads of b/q
whole sequences, so this is computed locally; the oracle simply loops over
every (sequence, head).

The 3h-wide projection output is ordered head-major: column
head*3d + {0: Q, 1: K, 2: V}*d + e, so that a column block of the grid holds
Q, K and V of the same heads.
"""
import numpy as np


def softmax_rows(S):
    m = S.max(axis=1, keepdims=True)
    e = np.exp(S - m)
    return e / e.sum(axis=1, keepdims=True)


def softmax_rows_backward(P, dP):
    """Gradient of the row soft-max: with P = softmax_rows(S) and dP the gradient with respect to P,
    dS = P * (dP - rowsum(dP * P))."""
    P = np.asarray(P, dtype=np.float64)
    dP = np.asarray(dP, dtype=np.float64)
    return P * (dP - (dP * P).sum(axis=1, keepdims=True))


def head_forward(Q, K, V, causal=True):
    """One (sequence, head). Returns O [s,d] and P [s,s]."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s, d = Q.shape
    S = (Q @ K.T) / np.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones((s, s), dtype=bool)), S, -np.inf)
    P = softmax_rows(S)
    return P @ V, P


def head_logsumexp(Q, K, causal=True):
    """Row-wise log-sum-exp of the scaled (and masked) scores of one (sequence, head):
    L_t = log sum_u exp(S_tu), so that the soft-max row is P_tu = exp(S_tu - L_t).  It is the one
    per-row number an attention that never stores P (the operator fusion the paper's conclusion
    proposes) keeps for the backward pass."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    s, d = Q.shape
    S = (Q @ K.T) / np.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones((s, s), dtype=bool)), S, -np.inf)
    m = S.max(axis=1)
    return m + np.log(np.exp(S - m[:, None]).sum(axis=1))


def head_backward(Q, K, V, P, dO):
    """Gradients for one (sequence, head).

    dV = P^T dO; dP = dO V^T; dS = P * (dP - rowsum(dP * P));
    dQ = dS K / sqrt(d); dK = dS^T Q / sqrt(d).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    d = Q.shape[1]
    dV = P.T @ dO
    dP = dO @ V.T
    dS = softmax_rows_backward(P, dP)
    dQ = dS @ K / np.sqrt(d)
    dK = dS.T @ Q / np.sqrt(d)
    return dQ, dK, dV


def split_qkv(qkv, b, s, n, seq, head):
    """Views of Q, K, V [s, d] for one (sequence, head) out of qkv [b*s, 3h]."""
    h3 = qkv.shape[1]
    d = h3 // (3 * n)
    rows = slice(seq * s, (seq + 1) * s)
    c0 = head * 3 * d
    return (qkv[rows, c0:c0 + d], qkv[rows, c0 + d:c0 + 2 * d], qkv[rows, c0 + 2 * d:c0 + 3 * d])


def forward(qkv, b, s, n, causal=True, keep_probs=True):
    """qkv [b*s, 3h] -> attn [b*s, h] (heads concatenated) and probs [b, n, s, s]."""
    qkv = np.asarray(qkv, dtype=np.float64)
    h = qkv.shape[1] // 3
    d = h // n
    out = np.empty((b * s, h))
    probs = np.empty((b, n, s, s)) if keep_probs else None
    for seq in range(b):
        for head in range(n):
            Q, K, V = split_qkv(qkv, b, s, n, seq, head)
            O, P = head_forward(Q, K, V, causal)
            out[seq * s:(seq + 1) * s, head * d:(head + 1) * d] = O
            if keep_probs:
                probs[seq, head] = P
    return out, probs


def logsumexp(qkv, b, s, n, causal=True):
    """qkv [b*s, 3h] -> L [b, n, s]: head_logsumexp of every (sequence, head)."""
    qkv = np.asarray(qkv, dtype=np.float64)
    out = np.empty((b, n, s))
    for seq in range(b):
        for head in range(n):
            Q, K, _ = split_qkv(qkv, b, s, n, seq, head)
            out[seq, head] = head_logsumexp(Q, K, causal)
    return out


def backward(qkv, d_attn, b, s, n, causal=True, probs=None):
    """d_attn [b*s, h] -> d_qkv [b*s, 3h].  Probabilities are recomputed in fp64 unless the saved
    ones ([b, n, s, s]) are passed in."""
    qkv = np.asarray(qkv, dtype=np.float64)
    d_attn = np.asarray(d_attn, dtype=np.float64)
    h = qkv.shape[1] // 3
    d = h // n
    d_qkv = np.empty_like(qkv)
    for seq in range(b):
        for head in range(n):
            Q, K, V = split_qkv(qkv, b, s, n, seq, head)
            P = probs[seq, head] if probs is not None else head_forward(Q, K, V, causal)[1]
            dO = d_attn[seq * s:(seq + 1) * s, head * d:(head + 1) * d]
            dQ, dK, dV = head_backward(Q, K, V, P, dO)
            rows = slice(seq * s, (seq + 1) * s)
            c0 = head * 3 * d
            d_qkv[rows, c0:c0 + d] = dQ
            d_qkv[rows, c0 + d:c0 + 2 * d] = dK
            d_qkv[rows, c0 + 2 * d:c0 + 3 * d] = dV
    return d_qkv
