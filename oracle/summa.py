"""The three matrix products (Section 2.4, Eq. 1-3, Algorithms 1-3).

SUMMA reaches exactly the ordinary matrix product (up to summation order), so
the oracle for a device's output block is the plain product of the
unpartitioned matrices in fp64, cut at block (i, j).  ``grid_*`` replay the
three algorithms step by step on q*q virtual devices (broadcast = read the
root's block, reduce = sum onto the root); they exist to pin the block index
formulas, not to be fast.
"""
import numpy as np

from . import blocks as _b


def f64(x):
    return np.asarray(x, dtype=np.float64)


# ---- plain definitions -----------------------------------------------------
def matmul_ab(A, B):
    """C = A B with A[M,K], B[K,N]."""
    return f64(A) @ f64(B)


def matmul_abt(A, B):
    """C = A B^T with A[M,K], B[N,K]."""
    return f64(A) @ f64(B).T


def matmul_atb(A, B):
    """C = A^T B with A[K,M], B[K,N]."""
    return f64(A).T @ f64(B)


def brute_matmul(form, A, B):
    """Triple loop in Python floats (fp64); for tiny inputs only."""
    A = f64(A)
    B = f64(B)
    if form == "ab":
        M, K = A.shape
        N = B.shape[1]
        a = lambda m, k: A[m, k]
        b = lambda k, n: B[k, n]
    elif form == "abt":
        M, K = A.shape
        N = B.shape[0]
        a = lambda m, k: A[m, k]
        b = lambda k, n: B[n, k]
    elif form == "atb":
        K, M = A.shape
        N = B.shape[1]
        a = lambda m, k: A[k, m]
        b = lambda k, n: B[k, n]
    else:
        raise ValueError(form)
    C = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += a(m, k) * b(k, n)
            C[m, n] = acc
    return C


# ---- gradients (Eq. 1-3) ---------------------------------------------------
def grads_ab(A, B, dC):
    """C = A B  ->  dA = dC B^T, dB = A^T dC   (Eq. 1)."""
    return matmul_abt(dC, B), matmul_atb(A, dC)


def grads_atb(A, B, dC):
    """C = A^T B  ->  dA = B dC^T, dB = A dC   (Eq. 2)."""
    return matmul_abt(B, dC), matmul_ab(A, dC)


def grads_abt(A, B, dC):
    """C = A B^T  ->  dA = dC B, dB = dC^T A   (Eq. 3)."""
    return matmul_ab(dC, B), matmul_atb(dC, A)


# ---- virtual-grid replays of Algorithms 1-3 --------------------------------
def grid_ab(Ab, Bb):
    """Algorithm 1 on q*q virtual devices. Ab, Bb: [q,q,.,.] blocks. Returns C blocks."""
    q = Ab.shape[0]
    Ab, Bb = f64(Ab), f64(Bb)
    Cb = np.zeros((q, q, Ab.shape[2], Bb.shape[3]))
    for l in range(q):
        for i in range(q):
            for j in range(q):
                a_recv = Ab[i, l]          # broadcast of A_il within row i (root: column l)
                b_recv = Bb[l, j]          # broadcast of B_lj within column j (root: row l)
                Cb[i, j] += a_recv @ b_recv
    return Cb


def grid_abt(Ab, Bb):
    """Algorithm 2: per step l every device (i,j) forms A_ij (B_lj)^T, row i reduces onto C_il."""
    q = Ab.shape[0]
    Ab, Bb = f64(Ab), f64(Bb)
    Cb = np.zeros((q, q, Ab.shape[2], Bb.shape[2]))
    for l in range(q):
        for i in range(q):
            acc = np.zeros((Ab.shape[2], Bb.shape[2]))
            for j in range(q):
                b_recv = Bb[l, j]          # broadcast of B_lj within column j
                acc += Ab[i, j] @ b_recv.T  # C^temp_ij, reduced within row i
            Cb[i, l] = acc                 # root of the reduce: device (i, l)
    return Cb


def grid_atb(Ab, Bb):
    """Algorithm 3: per step l every device (i,j) forms (A_il)^T B_ij, column j reduces onto C_lj."""
    q = Ab.shape[0]
    Ab, Bb = f64(Ab), f64(Bb)
    Cb = np.zeros((q, q, Ab.shape[3], Bb.shape[3]))
    for l in range(q):
        for j in range(q):
            acc = np.zeros((Ab.shape[3], Bb.shape[3]))
            for i in range(q):
                a_recv = Ab[i, l]          # broadcast of A_il within row i
                acc += a_recv.T @ Bb[i, j]  # C^temp_ij, reduced within column j
            Cb[l, j] = acc                 # root of the reduce: device (l, j)
    return Cb


# ---- owner view: what device (i, j) ends up holding ------------------------
def owner_block(form, A, B, q, i, j):
    """Block (i, j) of the product, written as the sum over the q panels the
    device consumes: AB: sum_l A_il B_lj; ABT: sum_l A_il (B_jl)^T;
    ATB: sum_l (A_li)^T B_lj."""
    A, B = f64(A), f64(B)
    acc = None
    for l in range(q):
        if form == "ab":
            t = _b.block(A, q, i, l) @ _b.block(B, q, l, j)
        elif form == "abt":
            t = _b.block(A, q, i, l) @ _b.block(B, q, j, l).T
        elif form == "atb":
            t = _b.block(A, q, l, i).T @ _b.block(B, q, l, j)
        else:
            raise ValueError(form)
        acc = t if acc is None else acc + t
    return acc


def product(form, A, B):
    return {"ab": matmul_ab, "abt": matmul_abt, "atb": matmul_atb}[form](A, B)
