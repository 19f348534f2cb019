"""Device-memory helpers for the benchmark and examples: upload row-major host arrays and bring them into the
library's block-major layout with the library's own pack kernel.  PyTorch is used for allocation only."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as opt

DEV = "cuda:0"


def upload_bf16_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns (any shape) -> flat bf16 device tensor."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).reshape(-1)).to(DEV).view(torch.bfloat16)


def pack_matrix(rowmajor: torch.Tensor, R: int, C: int, q: int) -> torch.Tensor:
    """flat row-major device tensor -> new flat block-major device tensor (optimus_pack_blocks)."""
    out = torch.empty_like(rowmajor)
    opt.pack_blocks(rowmajor, out, R, C, q, rowmajor.element_size())
    return out


LAYER_MATS = {
    "x": (1, 1), "w_qkv": (0, 3), "w_o": (0, 1), "w1": (0, 4), "w2": (4, 1), "d_out": (1, 1),
}


def layer_shapes(b, s, h):
    M = b * s
    return {
        "x": (M, h), "w_qkv": (h, 3 * h), "w_o": (h, h), "w1": (h, 4 * h), "w2": (4 * h, h), "d_out": (M, h),
        "ln1_out": (M, h), "xhat1": (M, h), "qkv": (M, 3 * h), "attn": (M, h), "h_mid": (M, h), "ln2_out": (M, h),
        "xhat2": (M, h), "pre_gelu": (M, 4 * h), "gelu": (M, 4 * h), "out": (M, h),
        "d_pre_gelu": (M, 4 * h), "d_ln2_out": (M, h), "d_h_mid": (M, h), "d_attn": (M, h), "d_qkv": (M, 3 * h),
        "d_ln1_out": (M, h), "d_x": (M, h),
        "d_w_qkv": (h, 3 * h), "d_w_o": (h, h), "d_w1": (h, 4 * h), "d_w2": (4 * h, h),
    }


def alloc_layer(inputs_bits: dict, vectors: dict, b, s, h, n, q, causal=True, eps=1e-5, fused_attention=False, share=None):
    """inputs_bits: name -> uint16 bf16 patterns of the six input matrices (row-major);
    vectors: name -> fp32 numpy vectors.  Returns (cfg, tensors dict, LayerTensors, workspace).
    With ``fused_attention`` the layer keeps lse [q][q][(b/q)(n/q)][s] instead of probs.  ``share``: a tensors dict
    of an earlier call whose inputs and parameters are reused instead of uploaded again."""
    shapes = layer_shapes(b, s, h)
    M = b * s
    T = {}
    for name in ("x", "w_qkv", "w_o", "w1", "w2", "d_out"):
        R, C = shapes[name]
        T[name] = share[name] if share is not None else pack_matrix(upload_bf16_bits(inputs_bits[name]), R, C, q)
    for name, v in vectors.items():
        T[name] = share[name] if share is not None else torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(DEV)
    for name, (R, C) in shapes.items():
        if name in T:
            continue
        dt = torch.float32 if name.startswith("d_w") else torch.bfloat16
        T[name] = torch.zeros(R * C, dtype=dt, device=DEV)
    rows = M // q
    nmat = (b // q) * (n // q)
    if fused_attention:
        T["lse"] = torch.zeros(q * q * nmat * s, dtype=torch.float32, device=DEV)
    else:
        T["probs"] = torch.zeros(q * q * nmat * s * s, dtype=torch.bfloat16, device=DEV)
    for name in ("rstd1", "rstd2"):
        T[name] = torch.zeros(q * q * rows, dtype=torch.float32, device=DEV)
    for name in ("stats1", "stats2", "bstats1", "bstats2"):
        T[name] = torch.zeros(q * q * rows * 2, dtype=torch.float32, device=DEV)
    for name, mult in {"d_b_qkv": 3, "d_b_o": 1, "d_b1": 4, "d_b2": 1, "d_ln1_g": 1, "d_ln1_b": 1, "d_ln2_g": 1, "d_ln2_b": 1}.items():
        T[name] = torch.zeros(q * q * (mult * h // q), dtype=torch.float32, device=DEV)
    cfg = opt.LayerCfg(b, s, h, n, q, eps, 1 if causal else 0, opt.BF16, 1 if fused_attention else 0)
    ws = torch.empty(opt.layer_workspace_bytes(cfg), dtype=torch.uint8, device=DEV)
    return cfg, T, opt.make_layer_tensors(T), ws
