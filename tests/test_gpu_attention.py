"""GPU parity: head-partitioned local attention (forward and backward) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import attention as oatt
from oracle.metrics import rel_frobenius
from workloads import round_to_bf16
from gpu_util import to_host, mat_to_dev, mat_to_host, empty

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _probs_blocks(probs, b, n, q):
    """oracle probs [b, n, s, s] -> [q, q, (b/q)*(n/q), s, s] in the library's device order."""
    nb, nh = b // q, n // q
    s = probs.shape[-1]
    out = np.empty((q, q, nb * nh, s, s))
    for i in range(q):
        for j in range(q):
            out[i, j] = probs[i * nb:(i + 1) * nb, j * nh:(j + 1) * nh].reshape(nb * nh, s, s)
    return out


# (b, s, h, n, q): several tiles per score matrix, ragged s (multiple of 8 only), d = 64 and 128, q = 1,
# config-4-like s = 1024 with d = 128, and the longest sequence the soft-max kernels accept (s = 4096)
CASES = [(4, 64, 64, 4, 2), (2, 328, 256, 2, 2), (2, 256, 128, 2, 1), (4, 136, 128, 8, 4), (2, 1024, 256, 2, 2),
         (1, 4096, 64, 1, 1)]


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("b,s,h,n,q", CASES)
def test_attention_forward_backward(b, s, h, n, q, causal):
    rng = np.random.default_rng(b * 1000 + s)
    M = b * s
    qkv = round_to_bf16(rng.standard_normal((M, 3 * h)).astype(np.float32))
    d_attn = round_to_bf16(rng.standard_normal((M, h)).astype(np.float32))
    attn_o, probs_o = oatt.forward(qkv, b, s, n, causal)
    dqkv_o = oatt.backward(qkv, d_attn, b, s, n, causal)

    nbytes = opt.attention_workspace_bytes(b, s, h, n, q)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    dQKV = mat_to_dev(qkv, q, "bf16")
    nmat = (b // q) * (n // q)
    P = empty(q * q * nmat * s * s, "bf16")
    O = empty(M * h, "bf16")
    opt.attention_fwd(dQKV, P, O, b, s, h, n, q, -1, -1, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    assert rel_frobenius(mat_to_host(O, M, h, q), attn_o) <= TOL
    p = to_host(P).reshape(q, q, nmat, s, s)
    want_p = _probs_blocks(probs_o, b, n, q)
    assert rel_frobenius(p, want_p) <= TOL
    assert np.allclose(p.sum(axis=-1), 1.0, atol=2e-2)            # rows sum to one (bf16 storage)
    if causal:
        iu = np.triu_indices(s, 1)
        assert np.all(p[..., iu[0], iu[1]] == 0.0)                  # exact zeros above the diagonal
        assert np.all(p[..., 0, 0] == 1.0)

    # backward from the oracle's probabilities rounded to storage, so that only the backward arithmetic is compared
    Pin = torch.from_numpy(round_to_bf16(want_p.astype(np.float32)).reshape(-1)).to("cuda:0").to(torch.bfloat16)
    dO = mat_to_dev(d_attn, q, "bf16")
    dQ = empty(M * 3 * h, "bf16")
    opt.attention_bwd(dQKV, Pin, dO, dQ, b, s, h, n, q, -1, -1, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    got = mat_to_host(dQ, M, 3 * h, q)
    assert rel_frobenius(got, dqkv_o) <= TOL
    # per component (Q, K, V gradients separately, so a weak one cannot hide behind a strong one)
    d = h // n
    cols = np.arange(3 * h)
    for part in range(3):
        sel = (cols // d) % 3 == part
        assert rel_frobenius(got[:, sel], dqkv_o[:, sel]) <= TOL, part

    # one device only: same bits for its blocks, nothing else written
    i, j = q - 1, 0
    O1, P1 = empty(M * h, "bf16"), empty(q * q * nmat * s * s, "bf16")
    opt.attention_fwd(dQKV, P1, O1, b, s, h, n, q, i, j, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    blk = (M // q) * (h // q)
    a, a1 = to_host(O), to_host(O1)
    sl = slice((i * q + j) * blk, (i * q + j + 1) * blk)
    assert np.array_equal(a[sl], a1[sl])
    mask = np.ones(M * h, dtype=bool)
    mask[sl] = False
    assert np.all(np.isnan(a1[mask]))


@pytest.mark.parametrize("b,s,h,n,q,devices", [(4, 136, 128, 8, 4, 16), (4, 136, 128, 8, 4, 5), (2, 328, 256, 2, 2, 3)])
def test_whole_grid_in_batches_of_devices_same_bits(b, s, h, n, q, devices):
    """With scratch for g devices a whole-grid call takes g devices per launch (g = all of them, or a count that
    leaves a shorter last group): forward and backward give the bits of the device-after-device run."""
    rng = np.random.default_rng(s + devices)
    M = b * s
    qkv = round_to_bf16(rng.standard_normal((M, 3 * h)).astype(np.float32))
    d_attn = round_to_bf16(rng.standard_normal((M, h)).astype(np.float32))
    dQKV, dO = mat_to_dev(qkv, q, "bf16"), mat_to_dev(d_attn, q, "bf16")
    nmat = (b // q) * (n // q)
    one = opt.attention_workspace_bytes(b, s, h, n, q)
    res = []
    for g in (1, devices):
        ws = torch.empty(g * one, dtype=torch.uint8, device="cuda:0")
        P, O, dQ = empty(q * q * nmat * s * s, "bf16"), empty(M * h, "bf16"), empty(M * 3 * h, "bf16")
        opt.attention_fwd(dQKV, P, O, b, s, h, n, q, -1, -1, True, opt.BF16, ws)
        opt.attention_bwd(dQKV, P, dO, dQ, b, s, h, n, q, -1, -1, True, opt.BF16, ws)
        torch.cuda.synchronize()
        res.append((P, O, dQ))
    for x, y in zip(res[0], res[1]):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
    assert not torch.isnan(res[1][2].float()).any()


def test_attention_closed_forms():
    """Q = 0 gives uniform weights over the visible prefix: O_t = mean(V_0..t); constant V gives O = V."""
    b, s, h, n, q = 2, 128, 64, 2, 1
    d = h // n
    rng = np.random.default_rng(3)
    qkv = rng.standard_normal((b * s, 3 * h)).astype(np.float32)
    cols = np.arange(3 * h)
    qkv[:, (cols // d) % 3 == 0] = 0.0
    qkv = round_to_bf16(qkv)
    ws = torch.empty(opt.attention_workspace_bytes(b, s, h, n, q), dtype=torch.uint8, device="cuda:0")
    P, O = empty(b * n * s * s, "bf16"), empty(b * s * h, "bf16")
    opt.attention_fwd(mat_to_dev(qkv, q, "bf16"), P, O, b, s, h, n, q, 0, 0, True, opt.BF16, ws)
    torch.cuda.synchronize()
    out = mat_to_host(O, b * s, h, q)
    for seq in range(b):
        for head in range(n):
            V = qkv[seq * s:(seq + 1) * s, head * 3 * d + 2 * d:head * 3 * d + 3 * d].astype(np.float64)
            want = np.cumsum(V, axis=0) / np.arange(1, s + 1)[:, None]
            assert rel_frobenius(out[seq * s:(seq + 1) * s, head * d:(head + 1) * d], want) <= TOL


def test_attention_errors():
    one = empty(16, "bf16")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    for args, code in [((3, 64, 64, 4, 2), opt.ESHAPE),     # b not divisible by q
                       ((4, 64, 64, 3, 2), opt.ESHAPE),     # n not divisible by q
                       ((4, 60, 64, 4, 2), opt.ESHAPE),     # s not a multiple of 8
                       ((4, 8192, 64, 4, 2), opt.ESHAPE)]:  # s beyond the documented limit
        with pytest.raises(opt.OptimusError) as e:
            opt.attention_fwd(one, one, one, *args, 0, 0, True, opt.BF16, ws)
        assert e.value.code == code
