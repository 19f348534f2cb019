"""GPU: the entry point that allocates nothing (optimus_attention_fused_bwd_static, scratch in a static device array)
against the existing entry point with a caller-provided workspace: same bits, on two calls in a row, the second with
a smaller input (the array keeps the first call's contents), in grid mode and for one device; and the size limit."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import attention as oatt
from oracle.metrics import rel_frobenius
from workloads import round_to_bf16
from gpu_util import mat_to_dev, mat_to_host, empty

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _case(b, s, h, n, q, causal, seed):
    rng = np.random.default_rng(seed)
    M = b * s
    qkv = round_to_bf16(rng.standard_normal((M, 3 * h)).astype(np.float32))
    d_attn = round_to_bf16(rng.standard_normal((M, h)).astype(np.float32))
    nmat = (b // q) * (n // q)
    dQKV, dO = mat_to_dev(qkv, q, "bf16"), mat_to_dev(d_attn, q, "bf16")
    O, L = empty(M * h, "bf16"), empty(q * q * nmat * s, "fp32")
    opt.attention_fused_fwd(dQKV, O, L, b, s, h, n, q, -1, -1, causal, opt.BF16)
    return dict(b=b, s=s, h=h, n=n, q=q, causal=causal, M=M, qkv=qkv, d_attn=d_attn, dQKV=dQKV, dO=dO, O=O, L=L)


def _both(c, i, j):
    """d_qkv from the existing entry point (workspace given) and from the allocation-free one."""
    b, s, h, n, q, causal = c["b"], c["s"], c["h"], c["n"], c["q"], c["causal"]
    ws = torch.empty(opt.attention_fused_workspace_bytes(b, s, h, n, q), dtype=torch.uint8, device="cuda:0")
    want = torch.zeros(c["M"] * 3 * h, dtype=torch.bfloat16, device="cuda:0")
    got = torch.zeros(c["M"] * 3 * h, dtype=torch.bfloat16, device="cuda:0")
    opt.attention_fused_bwd(c["dQKV"], c["O"], c["L"], c["dO"], want, b, s, h, n, q, i, j, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    opt.attention_fused_bwd_static(c["dQKV"], c["O"], c["L"], c["dO"], got, b, s, h, n, q, i, j, causal, opt.BF16)
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_two_calls_second_smaller():
    big = _case(4, 328, 256, 4, 2, True, 1)       # ragged s, head width 64, whole grid: 4 * 4 * 328 rows of scratch
    small = _case(2, 100, 256, 2, 2, False, 2)    # fewer and shorter matrices, head width 128
    for c, (i, j) in ((big, (-1, -1)), (small, (-1, -1)), (big, (1, 0)), (small, (0, 1))):
        print("no-alloc case", c["b"], c["s"], c["h"], c["n"], c["q"], c["causal"], (i, j), flush=True)
        want, got = _both(c, i, j)
        assert torch.equal(want.view(torch.int16), got.view(torch.int16))
        if (i, j) == (-1, -1):   # and both are the oracle's gradient
            dqkv_o = oatt.backward(c["qkv"], c["d_attn"], c["b"], c["s"], c["n"], c["causal"])
            assert rel_frobenius(mat_to_host(got, c["M"], 3 * c["h"], c["q"]), dqkv_o) <= TOL


def test_static_scratch_rejects_what_does_not_fit():
    assert opt.STATIC_SCRATCH_BYTES == 4 << 20
    one = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    lse = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    # one device of q = 1: 8 * 8 matrices of s = 16400 rows -> 4.2 MB of scratch: rejected before anything is enqueued
    with pytest.raises(opt.OptimusError) as e:
        opt.attention_fused_bwd_static(one, one, lse, one, one, 8, 16400, 512, 8, 1, 0, 0, True, opt.BF16)
    assert e.value.code == opt.EWORKSPACE
    with pytest.raises(opt.OptimusError) as e:
        opt.attention_fused_bwd_static(one, one, lse, one, one, 4, 64, 64, 4, 2, 0, 0, True, opt.BF16)   # head width 16
    assert e.value.code == opt.ESHAPE
    with pytest.raises(opt.OptimusError) as e:
        opt.attention_fused_bwd_static(None, one, lse, one, one, 4, 64, 256, 4, 2, 0, 0, True, opt.BF16)
    assert e.value.code == opt.EINVAL
