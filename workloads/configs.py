"""Shapes of the five benchmark configurations (sizes only, no data).

Each GEMM case names a logical product with OUTPUT shape [M, N] and
contraction length K on a q x q grid; one device's share is
[M/q, N/q] accumulated over q panels of width K/q.
"""
from __future__ import annotations

from dataclasses import dataclass

from .inputs import LayerShape


@dataclass(frozen=True)
class GemmCase:
    name: str
    form: str   # 'ab' | 'abt' | 'atb'
    M: int
    K: int
    N: int
    q: int
    dtype: str
    seed: int
    dist_a: str = "n1"
    dist_b: str = "n02"

    @property
    def flops_per_device(self) -> int:
        return 2 * (self.M // self.q) * self.K * (self.N // self.q)


def _linear_cases(prefix, Mrows, Kin, Nout, q, dtype, seed, forms=("ab", "abt", "atb")):
    """Forward product Y[M,N] = X[M,K] W[K,N] and its two gradient products."""
    out = []
    if "ab" in forms:   # Y = X W
        out.append(GemmCase(f"{prefix}.ab", "ab", Mrows, Kin, Nout, q, dtype, seed, "n1", "n02"))
    if "abt" in forms:  # dX[M,Kin] = dY[M,Nout] W[Kin,Nout]^T : output [M,Kin], contraction Nout
        out.append(GemmCase(f"{prefix}.abt", "abt", Mrows, Nout, Kin, q, dtype, seed + 100, "n1", "n02"))
    if "atb" in forms:  # dW[Kin,Nout] = X[M,Kin]^T dY[M,Nout] : output [Kin,Nout], contraction M
        out.append(GemmCase(f"{prefix}.atb", "atb", Kin, Mrows, Nout, q, dtype, seed + 200, "n1", "n1"))
    return out


CONFIGS = {
    # q=2, fp32, MLP up-projection b=2, s=16, h=64, all four device blocks.
    "config1": dict(q=2, dtype="fp32", seed=0, b=2, s=16, h=64),
    # q=4, bf16, BERT-Large-like layer b=8, s=512, h=1024, 16 heads.
    "config2": dict(q=4, dtype="bf16", seed=1, layer=LayerShape(b=8, s=512, h=1024, n=16, q=4)),
    # q=8, bf16 thin panels b=32, s=512, h=3072.
    "config3": dict(q=8, dtype="bf16", seed=2, b=32, s=512, h=3072),
    # q=4, bf16 full layer b=8, s=1024, h=4096, 32 heads, causal.
    "config4": dict(q=4, dtype="bf16", seed=3, layer=LayerShape(b=8, s=1024, h=4096, n=32, q=4)),
    # q=8, bf16 large batch b=64, s=512, h=4096, 32 heads.
    "config5": dict(q=8, dtype="bf16", seed=4, layer=LayerShape(b=64, s=512, h=4096, n=32, q=8)),
}


def gemm_cases(name: str):
    """SUMMA products of a configuration (logical shapes)."""
    if name == "config1":
        c = CONFIGS[name]
        M, h = c["b"] * c["s"], c["h"]
        cases = _linear_cases("mlp_up", M, h, 4 * h, c["q"], "fp32", c["seed"])
        # config 1 draws X, W uniform[-1,1] and the upstream gradient N(0,1)
        fixed = []
        for g in cases:
            da, db = {"ab": ("u", "u"), "abt": ("n1", "u"), "atb": ("u", "n1")}[g.form]
            fixed.append(GemmCase(g.name, g.form, g.M, g.K, g.N, g.q, g.dtype, g.seed, da, db))
        return fixed
    if name == "config2":
        c = CONFIGS[name]
        L = c["layer"]
        M, h, q, sd = L.M, L.h, L.q, c["seed"]
        return (_linear_cases("qkv", M, h, 3 * h, q, "bf16", sd)
                + _linear_cases("mlp_up", M, h, 4 * h, q, "bf16", sd + 1)
                + _linear_cases("mlp_down", M, 4 * h, h, q, "bf16", sd + 2))
    if name == "config3":
        c = CONFIGS[name]
        M, h, q, sd = c["b"] * c["s"], c["h"], c["q"], c["seed"]
        return (_linear_cases("mlp_up", M, h, 4 * h, q, "bf16", sd)
                + _linear_cases("mlp_down", M, 4 * h, h, q, "bf16", sd + 1))
    if name in ("config4", "config5"):
        c = CONFIGS[name]
        L = c["layer"]
        M, h, q, sd = L.M, L.h, L.q, c["seed"]
        return (_linear_cases("qkv", M, h, 3 * h, q, "bf16", sd)
                + _linear_cases("dense", M, h, h, q, "bf16", sd + 1)
                + _linear_cases("mlp_up", M, h, 4 * h, q, "bf16", sd + 2)
                + _linear_cases("mlp_down", M, 4 * h, h, q, "bf16", sd + 3))
    raise KeyError(name)
