"""The two ends of the model around the layer stack (Sections 3.2.1 and 3.2.2 of the paper): the
embedding of token indices, the lm-head logits, and the token-wise cross entropy.

Embedding: the paper views it as the product of the one-hot matrix [b*s, v] of the token
indices with the embedding table [v, h], which is the row gather ``table[tokens]``; its
gradient with respect to the table is one-hot^T times the output gradient (a scatter-add of
rows).  The lm-head multiplies the hidden states with the transposed table (the C = A B^T
product).  Cross entropy for one-hot targets: H = log(sum_i exp(x_i)) - x_l; the predicted
distribution is q_j = exp(x_j) / sum_i exp(x_i) (the formula as printed lacks the
exponential in the numerator; with it the stated gradient q_j - [j = l] is the derivative of
H, which the finite-difference pin confirms), and d H / d x_j = q_j - [j = l].

Test infrastructure only.
"""
import numpy as np


def one_hot(tokens, v):
    tokens = np.asarray(tokens).reshape(-1)
    out = np.zeros((tokens.size, v))
    out[np.arange(tokens.size), tokens] = 1.0
    return out


def embedding(tokens, table):
    """tokens [b*s] ints, table [v, h] -> [b*s, h]."""
    return np.asarray(table, dtype=np.float64)[np.asarray(tokens).reshape(-1)]


def embedding_grad(tokens, d_x, v):
    """d_table [v, h] = one_hot^T d_x: row r collects the output-gradient rows of the tokens equal to r."""
    tokens = np.asarray(tokens).reshape(-1)
    d_x = np.asarray(d_x, dtype=np.float64)
    out = np.zeros((v, d_x.shape[1]))
    for t in range(tokens.size):
        out[tokens[t]] += d_x[t]
    return out


def lm_head(hidden, table):
    """logits [b*s, v] = hidden [b*s, h] table^T."""
    return np.asarray(hidden, dtype=np.float64) @ np.asarray(table, dtype=np.float64).T


def cross_entropy(logits, labels):
    """Per-token loss H_t = log sum_i exp(x_ti) - x_t,label and the row log-sum-exp L_t."""
    x = np.asarray(logits, dtype=np.float64)
    labels = np.asarray(labels).reshape(-1)
    m = x.max(axis=1)
    lse = m + np.log(np.exp(x - m[:, None]).sum(axis=1))
    return lse - x[np.arange(x.shape[0]), labels], lse


def cross_entropy_grad(logits, labels, scale=1.0):
    """d(sum_t scale * H_t) / d logits = scale * (q - one_hot(label))."""
    x = np.asarray(logits, dtype=np.float64)
    _, lse = cross_entropy(x, labels)
    g = np.exp(x - lse[:, None])
    g[np.arange(x.shape[0]), np.asarray(labels).reshape(-1)] -= 1.0
    return scale * g
