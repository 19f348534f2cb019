"""Seeded input generators (no arithmetic of the method lives here).

Every tensor is drawn in fp64 from ``numpy.random.default_rng(seed)`` in a
fixed, documented order, cast to fp32 and, for the bf16 configurations,
rounded to bf16 (round-to-nearest-even) *before* either the oracle or the
HIP path sees it.  Both sides therefore start from bit-identical values and
the parity error measures arithmetic only, not input quantisation.

Values are returned as float32 numpy arrays holding exactly representable
numbers; ``bf16_bits`` gives the 16-bit patterns to upload.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result is fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(x.shape)
    nan = np.isnan(x)
    if nan.any():
        out = out.copy()
        out[nan] = np.float32(np.nan)
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """16-bit patterns of values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    if np.any(u & 0xFFFF):
        raise ValueError("bf16_bits: value is not bf16-representable; call round_to_bf16 first")
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Inverse of ``bf16_bits``: uint16 patterns -> fp32 values."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _store(x64: np.ndarray, dtype: str) -> np.ndarray:
    x = x64.astype(np.float32)
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "fp32":
        return x
    raise ValueError(f"unknown dtype {dtype!r}")


def _draw(rng, dist: str, shape):
    """dist: 'u' uniform[-1,1], 'n1' N(0,1), 'n02' N(0, std 0.02)."""
    if dist == "u":
        return rng.uniform(-1.0, 1.0, size=shape)
    if dist == "n1":
        return rng.standard_normal(size=shape)
    if dist == "n02":
        return 0.02 * rng.standard_normal(size=shape)
    raise ValueError(dist)


def gemm_inputs(seed: int, form: str, M: int, K: int, N: int, dtype: str,
                dist_a: str = "n1", dist_b: str = "n02"):
    """Operands of one logical product with OUTPUT shape [M, N] and contraction K.

    form 'ab' : A[M,K], B[K,N];  'abt': A[M,K], B[N,K];  'atb': A[K,M], B[K,N].
    Draw order: A then B, from one generator seeded with ``seed``.
    """
    rng = np.random.default_rng(seed)
    shape_a = {"ab": (M, K), "abt": (M, K), "atb": (K, M)}[form]
    shape_b = {"ab": (K, N), "abt": (N, K), "atb": (K, N)}[form]
    a = _store(_draw(rng, dist_a, shape_a), dtype)
    b = _store(_draw(rng, dist_b, shape_b), dtype)
    return a, b


@dataclass(frozen=True)
class LayerShape:
    b: int      # batch (sequences)
    s: int      # sequence length
    h: int      # hidden size
    n: int      # attention heads
    q: int      # SUMMA dimension (grid is q x q)

    @property
    def M(self) -> int:
        return self.b * self.s

    @property
    def d(self) -> int:
        return self.h // self.n


def layer_inputs(seed: int, shp: LayerShape, dtype: str = "bf16", perturb_affine: bool = False):
    """All inputs of one transformer layer, logical (unpartitioned, row-major) layout.

    Draw order (one generator): x, w_qkv, w_o, w1, w2, d_out, then — only when
    ``perturb_affine`` — b_qkv, b_o, b1, b2, ln1_g, ln1_b, ln2_g, ln2_b.
    Rows of x/d_out are ordered sequence-major (row = seq * s + t).  Without
    ``perturb_affine`` biases are 0, gammas 1, betas 0 (the benchmark recipe);
    tests perturb them so that every term of the formulas is exercised.
    """
    rng = np.random.default_rng(seed)
    M, h = shp.M, shp.h
    t = {}
    t["x"] = _store(_draw(rng, "n1", (M, h)), dtype)
    t["w_qkv"] = _store(_draw(rng, "n02", (h, 3 * h)), dtype)
    t["w_o"] = _store(_draw(rng, "n02", (h, h)), dtype)
    t["w1"] = _store(_draw(rng, "n02", (h, 4 * h)), dtype)
    t["w2"] = _store(_draw(rng, "n02", (4 * h, h)), dtype)
    t["d_out"] = _store(_draw(rng, "n1", (M, h)), dtype)
    vec = {"b_qkv": 3 * h, "b_o": h, "b1": 4 * h, "b2": h,
           "ln1_g": h, "ln1_b": h, "ln2_g": h, "ln2_b": h}
    for name, n in vec.items():
        if perturb_affine:
            v = 0.1 * rng.standard_normal(size=(n,))
            if name.endswith("_g"):
                v = 1.0 + v
        else:
            v = np.ones(n) if name.endswith("_g") else np.zeros(n)
        # vectors are stored in fp32 on the device but kept bf16-representable
        t[name] = _store(v, dtype)
    return t


def token_inputs(seed: int, b: int, s: int, v: int):
    """Token indices [b*s] (int32, sequence-major rows) and next-token labels [b*s] with the rank-frequency shape of
    text: index r is drawn with probability proportional to 1/(r + 1) (Zipf), so a few rows of the embedding table
    collect many gradient rows and most collect none."""
    rng = np.random.default_rng(seed)
    p = 1.0 / np.arange(1, v + 1)
    p /= p.sum()
    tokens = rng.choice(v, size=b * s, p=p).astype(np.int32)
    labels = rng.choice(v, size=b * s, p=p).astype(np.int32)
    return tokens, labels
