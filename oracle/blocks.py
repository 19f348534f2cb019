"""2D block partition of a matrix over a q x q grid (Section 2.4, SUMMA).

A matrix T[R, C] is split evenly into q x q sub-blocks; block (i, j) is rows
i*R/q .. (i+1)*R/q-1 and columns j*C/q .. (j+1)*C/q-1 and lives on device
(i, j).  The resident layout used by the library is block-major: the q*q
sub-blocks stored one after another, block (i, j) at index i*q + j, each
sub-block row-major.
"""
import numpy as np


def check_divisible(R, C, q):
    if q <= 0 or R % q or C % q:
        raise ValueError(f"[{R} x {C}] is not evenly divisible over a {q} x {q} grid")


def block(T, q, i, j):
    """Sub-block (i, j) of T, as a view."""
    R, C = T.shape
    check_divisible(R, C, q)
    r, c = R // q, C // q
    return T[i * r:(i + 1) * r, j * c:(j + 1) * c]


def partition(T, q):
    """All sub-blocks: array of shape [q, q, R/q, C/q] (copy)."""
    R, C = T.shape
    check_divisible(R, C, q)
    out = np.empty((q, q, R // q, C // q), dtype=T.dtype)
    for i in range(q):
        for j in range(q):
            out[i, j] = block(T, q, i, j)
    return out


def assemble(blocks):
    """Inverse of ``partition``."""
    q, q2, r, c = blocks.shape
    assert q == q2
    T = np.empty((q * r, q * c), dtype=blocks.dtype)
    for i in range(q):
        for j in range(q):
            T[i * r:(i + 1) * r, j * c:(j + 1) * c] = blocks[i, j]
    return T


def pack_block_major(T, q):
    """Row-major logical matrix -> flat block-major storage."""
    return partition(T, q).reshape(-1)


def unpack_block_major(flat, R, C, q):
    """Flat block-major storage -> row-major logical matrix."""
    check_divisible(R, C, q)
    return assemble(np.asarray(flat).reshape(q, q, R // q, C // q))


def vector_slice(v, q, j):
    """Slice j of a length-C vector split evenly over the q grid columns."""
    C = v.shape[0]
    if C % q:
        raise ValueError("vector length not divisible by q")
    c = C // q
    return v[j * c:(j + 1) * c]
