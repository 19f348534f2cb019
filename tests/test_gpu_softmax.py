"""GPU parity: the row soft-max kernels of local attention by themselves (optimus_softmax_rows / _bwd) against the
oracle's definitions: fp32 scores in, bf16 probabilities out; with the causal mask, exact zeros above the diagonal."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import attention as oatt
from oracle.metrics import rel_frobenius
from workloads import round_to_bf16
from gpu_util import to_dev, to_host, empty

pytestmark = pytest.mark.gpu
TOL = 5e-3   # bf16 output of an fp32 computation


def _masked(S, causal):
    s = S.shape[-1]
    return np.where(np.tril(np.ones((s, s), dtype=bool)), S, -np.inf) if causal else S


# several rows per workgroup and a ragged last workgroup (nmat * s not a multiple of 4 rows per workgroup is
# impossible with s % 4 == 0, so ragged = the last lanes of a row: s = 100, 260), every register-count variant
# (s <= 256, 512, 1024, 2048, 4096), the benchmark sizes (s = 512 and 1024)
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("nmat,s", [(3, 4), (2, 100), (5, 260), (2, 512), (2, 1024), (1, 2048), (1, 4096)])
def test_softmax_rows_forward_backward(nmat, s, causal):
    rng = np.random.default_rng(nmat * 10000 + s)
    S = (rng.standard_normal((nmat, s, s)) * 1.6).astype(np.float32)
    dP = rng.standard_normal((nmat, s, s)).astype(np.float32)
    P_o = np.stack([oatt.softmax_rows(_masked(S[m].astype(np.float64), causal)) for m in range(nmat)])
    dS_dev, P_dev = empty(nmat * s * s, "bf16"), empty(nmat * s * s, "bf16")
    opt.softmax_rows(to_dev(S, "fp32"), P_dev, nmat, s, causal)
    torch.cuda.synchronize()
    P = to_host(P_dev).reshape(nmat, s, s)
    assert rel_frobenius(P, P_o) <= TOL
    if causal:
        iu = np.triu_indices(s, 1)
        assert np.all(P[:, iu[0], iu[1]] == 0.0)
    assert np.allclose(P.sum(axis=-1), 1.0, atol=2e-2)
    # backward from the oracle's probabilities rounded to the storage type, so that only the backward arithmetic differs
    P_in = round_to_bf16(P_o.astype(np.float32))
    dP_m = np.where(np.tril(np.ones((s, s), dtype=bool)), dP, 0.0) if causal else dP
    dS_o = np.stack([oatt.softmax_rows_backward(P_in[m], dP_m[m]) for m in range(nmat)])
    opt.softmax_rows_bwd(to_dev(dP, "fp32"), to_dev(P_in, "bf16"), dS_dev, nmat, s, causal)
    torch.cuda.synchronize()
    dS = to_host(dS_dev).reshape(nmat, s, s)
    assert rel_frobenius(dS, dS_o) <= TOL
    if causal:
        assert np.all(dS[:, iu[0], iu[1]] == 0.0)


def test_softmax_rows_closed_forms_and_errors():
    s, nmat = 64, 2
    # equal logits: row t of the causal soft-max is 1/(t+1) on columns <= t
    P_dev = empty(nmat * s * s, "bf16")
    opt.softmax_rows(torch.zeros(nmat * s * s, dtype=torch.float32, device="cuda:0"), P_dev, nmat, s, True)
    torch.cuda.synchronize()
    P = to_host(P_dev).reshape(nmat, s, s)
    want = np.tril(np.ones((s, s))) / np.arange(1, s + 1)[:, None]
    assert rel_frobenius(P[0], want) <= TOL and rel_frobenius(P[1], want) <= TOL
    # very large logits do not overflow (the row maximum is subtracted)
    big = torch.full((nmat * s * s,), 3.0e4, dtype=torch.float32, device="cuda:0")
    opt.softmax_rows(big, P_dev, nmat, s, False)
    torch.cuda.synchronize()
    assert rel_frobenius(to_host(P_dev), np.full(nmat * s * s, 1.0 / s)) <= TOL
    for bad_s in (0, 6, 4100):
        with pytest.raises(opt.OptimusError) as e:
            opt.softmax_rows(big, P_dev, 1, bad_s, True)
        assert e.value.code == opt.ESHAPE
    with pytest.raises(opt.OptimusError) as e:
        opt.softmax_rows(None, P_dev, 1, 64, True)
    assert e.value.code == opt.EINVAL
