"""GPU parity: Algorithms 1-3 replayed step by step from the computing device (per-step partial blocks in memory,
then the reduce onto the root), against the oracle's virtual-grid replays and the plain products, and against the
library's own fused owner-view entry points."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import blocks, summa
from oracle.metrics import rel_frobenius
from workloads import gemm_inputs
from gpu_util import mat_to_dev, mat_to_host, to_host, empty, dt

pytestmark = pytest.mark.gpu
TOL = {"bf16": 5e-3, "fp32": 1e-5}


def _operand_shapes(form, M, K, N):
    return {"ab": ((M, K), (K, N)), "abt": ((M, K), (N, K)), "atb": ((K, M), (K, N))}[form]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("form", ["ab", "abt", "atb"])
@pytest.mark.parametrize("q,M,K,N", [(2, 256, 128, 192), (4, 512, 256, 384), (4, 96, 160, 224)])
def test_algorithms_replayed_step_by_step(form, q, M, K, N, dtype):
    A, B = gemm_inputs(q * 100 + M, form, M, K, N, dtype, "n1", "n1")
    dA, dB = mat_to_dev(A, q, dtype), mat_to_dev(B, q, dtype)
    Mb, Nb = M // q, N // q
    C = empty(M * N, dtype)
    temps = empty(q * Mb * Nb, "fp32")
    want_blocks = {"ab": summa.grid_ab, "abt": summa.grid_abt, "atb": summa.grid_atb}[form](
        blocks.partition(np.asarray(A, dtype=np.float64), q), blocks.partition(np.asarray(B, dtype=np.float64), q))
    Ab, Bb = blocks.partition(np.asarray(A, dtype=np.float64), q), blocks.partition(np.asarray(B, dtype=np.float64), q)
    worst_partial = 0.0
    for l in range(q):
        for r in range(q):          # the row (ABT) / column (ATB) / device row (AB) whose reduce this is
            for k in range(q):      # the reducing index
                if form == "ab":    # device (r, k) accumulates its own C_rk over l: one partial per step
                    continue
                i, j = (r, k) if form == "abt" else (k, r)
                slot = temps[k * Mb * Nb:(k + 1) * Mb * Nb]
                opt.summa_step(form, dA, dB, slot, M, K, N, q, i, j, l, dt(dtype))
                torch.cuda.synchronize()
                want = Ab[i, j] @ Bb[l, j].T if form == "abt" else Ab[i, l].T @ Bb[i, j]
                worst_partial = max(worst_partial, rel_frobenius(to_host(slot).reshape(Mb, Nb), want))
            if form == "abt":
                opt.summa_reduce(temps, q, C, M, N, q, r, l, dt(dtype))     # root of row r's reduce: device (r, l)
            elif form == "atb":
                opt.summa_reduce(temps, q, C, M, N, q, l, r, dt(dtype))     # root of column r's reduce: device (l, r)
    if form == "ab":                # Algorithm 1: device (i, j) adds A_il B_lj over the steps
        for i in range(q):
            for j in range(q):
                for l in range(q):
                    slot = temps[l * Mb * Nb:(l + 1) * Mb * Nb]
                    opt.summa_step(form, dA, dB, slot, M, K, N, q, i, j, l, dt(dtype))
                    torch.cuda.synchronize()
                    worst_partial = max(worst_partial, rel_frobenius(to_host(slot).reshape(Mb, Nb), Ab[i, l] @ Bb[l, j]))
                opt.summa_reduce(temps, q, C, M, N, q, i, j, dt(dtype))
    torch.cuda.synchronize()
    got = mat_to_host(C, M, N, q)
    assert worst_partial <= TOL[dtype]
    assert rel_frobenius(got, summa.product(form, A, B)) <= TOL[dtype]
    assert rel_frobenius(blocks.partition(got.astype(np.float64), q), want_blocks) <= TOL[dtype]
    # the fused owner-view entry point computes the same matrix (other summation order)
    C2 = empty(M * N, dtype)
    opt.summa(form, dA, dB, C2, M, K, N, q, -1, -1, dt(dtype))
    torch.cuda.synchronize()
    assert rel_frobenius(got, mat_to_host(C2, M, N, q)) <= TOL[dtype]


def test_step_errors():
    one = empty(64, "bf16")
    t = empty(64, "fp32")
    with pytest.raises(opt.OptimusError) as e:
        opt.summa_step("abt", one, one, t, 32, 64, 256, 2, 0, 0, 2, opt.BF16)
    assert e.value.code == opt.ECOORD
    with pytest.raises(opt.OptimusError) as e:
        opt.summa_step("abt", one, one, t, 33, 64, 256, 2, 0, 0, 1, opt.BF16)
    assert e.value.code == opt.ESHAPE
    with pytest.raises(opt.OptimusError) as e:
        opt.summa_reduce(t, 0, one, 32, 64, 2, 0, 0, opt.BF16)
    assert e.value.code == opt.ESHAPE
