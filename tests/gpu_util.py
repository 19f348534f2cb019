"""Helpers for the GPU parity tests: host<->device transfer of block-major tensors.

Packing to block-major is done on the host with the oracle's block partition, so the GPU path's own
block addressing is checked against an independent implementation.
"""
import numpy as np
import torch

from oracle import blocks
from workloads import bf16_bits, bits_to_f32

DEV = "cuda:0"


def to_dev(x, dtype):
    """numpy fp32 (bf16-representable when dtype == 'bf16') -> flat device tensor."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return torch.from_numpy(bf16_bits(x).view(np.int16).reshape(-1)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(x.reshape(-1)).to(DEV)


def to_host(t):
    """flat device tensor -> numpy fp32."""
    if t.dtype == torch.bfloat16:
        return bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.float().cpu().numpy()


def mat_to_dev(T, q, dtype):
    """logical row-major matrix -> block-major device tensor."""
    return to_dev(blocks.pack_block_major(np.asarray(T, dtype=np.float32), q), dtype)


def mat_to_host(t, R, C, q):
    """block-major device tensor -> logical row-major numpy fp32."""
    return blocks.unpack_block_major(to_host(t), R, C, q)


def vec_to_dev(v):
    return torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(DEV)


def empty(n, dtype):
    td = {"bf16": torch.bfloat16, "fp32": torch.float32}[dtype]
    # filled with NaN so that unwritten outputs are caught
    return torch.full((int(n),), float("nan"), dtype=td, device=DEV)


def dt(dtype):
    return {"fp32": 0, "bf16": 1}[dtype]
