"""Pins for oracle/attention.py: brute-force loops, closed forms, finite differences."""
import math

import numpy as np

from oracle import attention as att


def _brute_head(Q, K, V, causal):
    s, d = Q.shape
    O = np.zeros((s, d))
    P = np.zeros((s, s))
    for t in range(s):
        last = t if causal else s - 1
        sc = [sum(Q[t, e] * K[u, e] for e in range(d)) / math.sqrt(d) for u in range(last + 1)]
        mx = max(sc)
        ex = [math.exp(v - mx) for v in sc]
        Z = sum(ex)
        for u in range(last + 1):
            P[t, u] = ex[u] / Z
            for e in range(d):
                O[t, e] += P[t, u] * V[u, e]
    return O, P


def test_head_forward_brute_force():
    rng = np.random.default_rng(0)
    Q, K, V = (rng.standard_normal((6, 4)) for _ in range(3))
    for causal in (True, False):
        O, P = att.head_forward(Q, K, V, causal)
        Ob, Pb = _brute_head(Q, K, V, causal)
        assert np.allclose(O, Ob, atol=1e-13) and np.allclose(P, Pb, atol=1e-13)


def test_closed_forms():
    rng = np.random.default_rng(1)
    s, d = 7, 4
    Q, K, V = (rng.standard_normal((s, d)) for _ in range(3))
    O, P = att.head_forward(Q, K, V, causal=True)
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-14)
    assert np.all(np.triu(P, 1) == 0.0)                      # exact zeros above the diagonal
    assert P[0, 0] == 1.0 and np.allclose(O[0], V[0])
    O0, _ = att.head_forward(np.zeros_like(Q), K, V, causal=True)
    prefix_mean = np.cumsum(V, axis=0) / np.arange(1, s + 1)[:, None]
    assert np.allclose(O0, prefix_mean, atol=1e-14)           # Q = 0 -> uniform weights
    Vc = np.tile(rng.standard_normal((1, d)), (s, 1))
    Oc, _ = att.head_forward(Q, K, Vc, causal=True)
    assert np.allclose(Oc, Vc, atol=1e-14)                    # constant V -> O = V


def test_qkv_layout_head_major():
    b, s, n, d = 2, 3, 2, 4
    h = n * d
    qkv = np.arange(b * s * 3 * h, dtype=np.float64).reshape(b * s, 3 * h)
    Q, K, V = att.split_qkv(qkv, b, s, n, seq=1, head=1)
    assert Q[0, 0] == qkv[1 * s + 0, 1 * 3 * d + 0]
    assert K[2, 1] == qkv[1 * s + 2, 1 * 3 * d + d + 1]
    assert V[1, 3] == qkv[1 * s + 1, 1 * 3 * d + 2 * d + 3]


def test_full_forward_is_per_head_loop_and_backward_fd():
    rng = np.random.default_rng(2)
    b, s, n, d = 2, 4, 2, 3
    h = n * d
    qkv = rng.standard_normal((b * s, 3 * h))
    R = rng.standard_normal((b * s, h))
    out, probs = att.forward(qkv, b, s, n, causal=True)
    Q, K, V = att.split_qkv(qkv, b, s, n, 1, 0)
    Ob, Pb = _brute_head(Q, K, V, True)
    assert np.allclose(out[s:2 * s, 0:d], Ob, atol=1e-13) and np.allclose(probs[1, 0], Pb, atol=1e-13)
    dqkv = att.backward(qkv, R, b, s, n, causal=True)
    hstep = 1e-6
    for idx in np.ndindex(*qkv.shape):
        p, m = qkv.copy(), qkv.copy()
        p[idx] += hstep
        m[idx] -= hstep
        fd = (np.sum(R * att.forward(p, b, s, n, True, False)[0]) - np.sum(R * att.forward(m, b, s, n, True, False)[0])) / (2 * hstep)
        assert abs(fd - dqkv[idx]) < 1e-6, idx


def test_logsumexp_closed_forms_brute_force_and_library():
    """L_t = log sum_u exp(S_tu): brute force, Q = 0 (L_t = log of the number of visible keys),
    all keys equal, scipy's logsumexp on independently built scores, and P = exp(S - L)."""
    from scipy.special import logsumexp as sp_lse
    rng = np.random.default_rng(3)
    s, d = 9, 4
    Q, K, V = (rng.standard_normal((s, d)) for _ in range(3))
    for causal in (True, False):
        L = att.head_logsumexp(Q, K, causal)
        for t in range(s):
            last = t if causal else s - 1
            sc = [sum(Q[t, e] * K[u, e] for e in range(d)) / math.sqrt(d) for u in range(last + 1)]
            assert abs(L[t] - math.log(sum(math.exp(v) for v in sc))) < 1e-12
        S = np.einsum("te,ue->tu", Q, K) / math.sqrt(d)
        if causal:
            S[np.triu_indices(s, 1)] = -np.inf
        assert np.allclose(L, sp_lse(S, axis=1), atol=1e-13)
        _, P = att.head_forward(Q, K, V, causal)
        with np.errstate(divide="ignore"):
            assert np.allclose(np.exp(S - L[:, None]), P, atol=1e-14)
        L0 = att.head_logsumexp(np.zeros_like(Q), K, causal)
        want = np.log(np.arange(1, s + 1)) if causal else np.full(s, math.log(s))
        assert np.allclose(L0, want, atol=1e-14)
    # all keys equal: every visible score of row t is the same number c_t -> L_t = c_t + log(#visible)
    Kc = np.tile(rng.standard_normal((1, d)), (s, 1))
    c = Q @ Kc[0] / math.sqrt(d)
    assert np.allclose(att.head_logsumexp(Q, Kc, True), c + np.log(np.arange(1, s + 1)), atol=1e-13)
    # the [b, n, s] wrapper is the per-head loop
    b, n = 2, 2
    qkv = rng.standard_normal((b * s, 3 * n * d))
    Lall = att.logsumexp(qkv, b, s, n, True)
    Qh, Kh, _ = att.split_qkv(qkv, b, s, n, 1, 0)
    assert Lall.shape == (b, n, s) and np.array_equal(Lall[1, 0], att.head_logsumexp(Qh, Kh, True))


def test_backward_row_term_equals_output_form():
    """rowsum(dP * P) = rowsum(dO * O): the identity that lets a backward pass without saved P use the saved
    output instead; and the gradients from probabilities rebuilt as exp(S - L) equal the oracle's."""
    rng = np.random.default_rng(4)
    s, d = 8, 5
    Q, K, V, dO = (rng.standard_normal((s, d)) for _ in range(4))
    for causal in (True, False):
        O, P = att.head_forward(Q, K, V, causal)
        dP = dO @ V.T
        assert np.allclose((dP * P).sum(axis=1), (dO * O).sum(axis=1), atol=1e-13)
        S = Q @ K.T / math.sqrt(d)
        if causal:
            S[np.triu_indices(s, 1)] = -np.inf
        with np.errstate(divide="ignore"):
            P2 = np.exp(S - att.head_logsumexp(Q, K, causal)[:, None])
        for a_, b_ in zip(att.head_backward(Q, K, V, P, dO), att.head_backward(Q, K, V, P2, dO)):
            assert np.allclose(a_, b_, atol=1e-13)


def test_softmax_rows_backward_finite_differences():
    """dS = P * (dP - rowsum(dP * P)) is the gradient of <R, softmax_rows(S)> (central differences in fp64)."""
    rng = np.random.default_rng(5)
    S = rng.standard_normal((5, 7))
    R = rng.standard_normal((5, 7))
    got = att.softmax_rows_backward(att.softmax_rows(S), R)
    eps = 1e-6
    for (r, c) in [(0, 0), (2, 3), (4, 6), (1, 5)]:
        Sp, Sm = S.copy(), S.copy()
        Sp[r, c] += eps
        Sm[r, c] -= eps
        fd = (np.sum(R * att.softmax_rows(Sp)) - np.sum(R * att.softmax_rows(Sm))) / (2 * eps)
        assert abs(fd - got[r, c]) < 1e-8
    # each row of dS sums to zero (a soft-max row is invariant to adding a constant to its logits)
    assert np.allclose(got.sum(axis=1), 0.0, atol=1e-14)
