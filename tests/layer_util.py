"""Allocation of the layer's device tensors and comparison with the oracle (shared by tests, smoke and bench)."""
import numpy as np
import torch

import paper_2104_05343_amd as opt
from oracle import blocks
from oracle.metrics import rel_frobenius
from gpu_util import mat_to_dev, mat_to_host, to_host, vec_to_dev

# Bound on the relative Frobenius error against the exact (fp64, nothing rounded) oracle of the whole layer.
TOL = 5e-3
# Gradients that lie behind the soft-max logits.  The two bf16 operands that feed the logits (LayerNorm-1 output
# into the QKV product, Q and K into QK^T) each carry one bf16 rounding (2^-9 relative, uniform); in the logit
# S = q.k / sqrt(d) that becomes an ABSOLUTE error of about 1.1e-3 * |q||k| / sqrt(d) per operand, and an absolute
# error of a logit is a RELATIVE error of its probability.  At the benchmark layers' logit scale (standard
# deviation 1.6) these two roundings alone put 5.3e-3 on the gradients behind the attention in an fp64 simulation
# that does nothing but round stored tensors, and 7.1-7.6e-3 once every stored tensor is rounded
# (oracle/rounding_study.py, tests/test_oracle_rounding_study.py): no kernel that feeds bf16 operands to the
# matrix cores can meet 5e-3 there.  Measured on the GPU against the exact oracle, whole tensors: configuration 4
# d_ln1_g 7.6e-3, d_ln1_out 7.6e-3, d_w_qkv 7.4e-3, d_qkv 7.4e-3, d_w_o 6.1e-3, d_x 5.5e-3; configuration 5
# d_ln1_out 7.5e-3; configuration 2 <= 4.7e-3.  These tensors are held to the largest measured value plus a
# margin (9e-3); every other tensor is held to TOL (configuration 4: attn 4.9e-3, all others <= 4.5e-3).
BEHIND_LOGITS = ("d_qkv", "d_ln1_out", "d_x", "d_w_qkv", "d_b_qkv", "d_w_o", "d_ln1_g", "d_ln1_b")
TOL_BEHIND_LOGITS = 9e-3


def bound(name):
    return TOL_BEHIND_LOGITS if name in BEHIND_LOGITS else TOL

MAT_SHAPES = {  # name -> (rows, cols) in units of (M, h): callables of (M, h)
    "x": lambda M, h: (M, h), "w_qkv": lambda M, h: (h, 3 * h), "w_o": lambda M, h: (h, h),
    "w1": lambda M, h: (h, 4 * h), "w2": lambda M, h: (4 * h, h), "d_out": lambda M, h: (M, h),
    "ln1_out": lambda M, h: (M, h), "xhat1": lambda M, h: (M, h), "qkv": lambda M, h: (M, 3 * h),
    "attn": lambda M, h: (M, h), "h_mid": lambda M, h: (M, h), "ln2_out": lambda M, h: (M, h),
    "xhat2": lambda M, h: (M, h), "pre_gelu": lambda M, h: (M, 4 * h), "gelu": lambda M, h: (M, 4 * h),
    "out": lambda M, h: (M, h), "d_pre_gelu": lambda M, h: (M, 4 * h), "d_ln2_out": lambda M, h: (M, h),
    "d_h_mid": lambda M, h: (M, h), "d_attn": lambda M, h: (M, h), "d_qkv": lambda M, h: (M, 3 * h),
    "d_ln1_out": lambda M, h: (M, h), "d_x": lambda M, h: (M, h),
    "d_w_qkv": lambda M, h: (h, 3 * h), "d_w_o": lambda M, h: (h, h), "d_w1": lambda M, h: (h, 4 * h),
    "d_w2": lambda M, h: (4 * h, h),
}
INPUT_MATS = ["x", "w_qkv", "w_o", "w1", "w2", "d_out"]
INPUT_VECS = ["ln1_g", "ln1_b", "b_qkv", "b_o", "ln2_g", "ln2_b", "b1", "b2"]
FP32_MATS = ["d_w_qkv", "d_w_o", "d_w1", "d_w2"]
VEC_PART = {"d_b_qkv": 3, "d_b_o": 1, "d_b1": 4, "d_b2": 1, "d_ln1_g": 1, "d_ln1_b": 1, "d_ln2_g": 1, "d_ln2_b": 1}
FWD_OUT = ["ln1_out", "xhat1", "qkv", "attn", "h_mid", "ln2_out", "xhat2", "pre_gelu", "gelu", "out"]
BWD_OUT = ["d_pre_gelu", "d_ln2_out", "d_h_mid", "d_attn", "d_qkv", "d_ln1_out", "d_x"]


def alloc_layer(inp, shp, causal=True, eps=1e-5, fill=float("nan"), fused=False):
    """Upload inputs (block-major) and allocate every other tensor of optimus_layer_tensors.  With ``fused`` the
    layer uses the attention that keeps no [s x s] tensor: no ``probs`` is allocated, ``lse`` is."""
    M, h, q = shp.M, shp.h, shp.q
    dev = "cuda:0"
    T = {}
    for name in INPUT_MATS:
        T[name] = mat_to_dev(inp[name], q, "bf16")
    for name in INPUT_VECS:
        T[name] = vec_to_dev(inp[name])
    for name, fn in MAT_SHAPES.items():
        if name in T:
            continue
        r, c = fn(M, h)
        T[name] = torch.full((r * c,), fill, dtype=torch.float32 if name in FP32_MATS else torch.bfloat16, device=dev)
    rows = M // q
    nmat = (shp.b // q) * (shp.n // q)
    if fused:
        T["lse"] = torch.full((q * q * nmat * shp.s,), fill, dtype=torch.float32, device=dev)
    else:
        T["probs"] = torch.full((q * q * nmat * shp.s * shp.s,), fill, dtype=torch.bfloat16, device=dev)
    for name in ("rstd1", "rstd2"):
        T[name] = torch.full((q * q * rows,), fill, dtype=torch.float32, device=dev)
    for name in ("stats1", "stats2", "bstats1", "bstats2"):
        T[name] = torch.full((q * q * rows * 2,), fill, dtype=torch.float32, device=dev)
    for name, mult in VEC_PART.items():
        T[name] = torch.full((q * q * (mult * h // q),), fill, dtype=torch.float32, device=dev)
    cfg = opt.LayerCfg(shp.b, shp.s, shp.h, shp.n, shp.q, eps, 1 if causal else 0, opt.BF16, 1 if fused else 0)
    ws = torch.empty(opt.layer_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
    return cfg, T, opt.make_layer_tensors(T), ws


def fetch(T, name, shp):
    """Device tensor -> logical numpy array (matrices unpacked from block-major)."""
    M, h, q = shp.M, shp.h, shp.q
    if name in MAT_SHAPES:
        r, c = MAT_SHAPES[name](M, h)
        return mat_to_host(T[name], r, c, q)
    return to_host(T[name])


def oracle_vec_partials(name, g_or, fwd_or, inp, shp):
    """Per-device partial [q, q, N/q] of a vector gradient: column sums over the device's rows only."""
    M, h, q = shp.M, shp.h, shp.q
    src = {"d_b_qkv": g_or["d_qkv"], "d_b_o": g_or["d_h_mid"], "d_b1": g_or["d_pre_gelu"], "d_b2": np.asarray(inp["d_out"], dtype=np.float64),
           "d_ln1_b": g_or["d_ln1_out"], "d_ln2_b": g_or["d_ln2_out"],
           "d_ln1_g": g_or["d_ln1_out"] * fwd_or["xhat1"], "d_ln2_g": g_or["d_ln2_out"] * fwd_or["xhat2"]}[name]
    N = src.shape[1]
    out = np.empty((q, q, N // q))
    for i in range(q):
        for j in range(q):
            out[i, j] = blocks.block(src, q, i, j).sum(axis=0)
    return out


def compare_all(T, shp, inp, fwd_o, bwd_o, bound_of=bound, check=True):
    """Every forward tensor, activation gradient, parameter gradient (per-device partials for the vectors) and
    LayerNorm statistic of a grid-mode run against the oracle's tensors: {name: relative Frobenius error}."""
    worst = {}
    for name in FWD_OUT:
        worst[name] = rel_frobenius(fetch(T, name, shp), fwd_o[name])
    for name in BWD_OUT + FP32_MATS:
        worst[name] = rel_frobenius(fetch(T, name, shp), bwd_o[name])
    q, rows = shp.q, shp.M // shp.q
    for k in ("1", "2"):
        r = to_host(T["rstd" + k]).reshape(q, q, rows)
        want = fwd_o["rstd" + k].reshape(q, 1, rows).repeat(q, axis=1)
        worst["rstd" + k] = rel_frobenius(r, want)
    for name in VEC_PART:
        got = to_host(T[name]).reshape(q, q, -1)
        worst[name] = rel_frobenius(got, oracle_vec_partials(name, bwd_o, fwd_o, inp, shp))
    if check:
        bad = {k: (v, bound_of(k)) for k, v in worst.items() if not (v <= bound_of(k))}
        assert not bad, f"over the bound (error, bound): {bad}\nall: {worst}"
    return worst
