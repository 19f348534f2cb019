"""GPU parity: attention without the [s x s] tensors (forward, log-sum-exp, backward) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import attention as oatt
from oracle.metrics import rel_frobenius
from workloads import round_to_bf16
from gpu_util import to_host, mat_to_dev, mat_to_host, empty

pytestmark = pytest.mark.gpu
TOL = 5e-3        # bf16 inputs and outputs, fp32 accumulation
TOL_LSE = 1e-5    # the row log-sum-exp is an fp32 result of exact bf16 products accumulated in fp32


def _lse_blocks(L, b, n, q):
    """oracle L [b, n, s] -> [q, q, (b/q)*(n/q), s] in the library's device order."""
    nb, nh = b // q, n // q
    s = L.shape[-1]
    out = np.empty((q, q, nb * nh, s))
    for i in range(q):
        for j in range(q):
            out[i, j] = L[i * nb:(i + 1) * nb, j * nh:(j + 1) * nh].reshape(nb * nh, s)
    return out


# (b, s, h, n, q): head widths 64 and 128; s below one 128-row tile, ragged (not a multiple of 64, 32 or 8), several
# tiles, q = 1, config-2- and config-4-like sequence lengths, and a sequence longer than the unfused path accepts
CASES = [(4, 64, 256, 4, 2), (2, 328, 256, 2, 2), (2, 256, 128, 2, 1), (4, 136, 256, 4, 4), (2, 100, 128, 2, 2),
         (2, 33, 256, 2, 1), (2, 512, 128, 2, 2), (2, 1024, 256, 2, 2), (1, 4360, 64, 1, 1),
         # many (sequence, head) pairs, ragged s
         (8, 392, 512, 8, 1), (8, 520, 1024, 8, 1),
         # enough work that the forward switches to 128-row workgroups of eight wavefronts (ragged and exact s)
         (8, 1024, 512, 8, 1), (8, 1100, 1024, 8, 1)]


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("b,s,h,n,q", CASES)
def test_fused_attention_forward_backward(b, s, h, n, q, causal):
    rng = np.random.default_rng(b * 1000 + s + 7)
    M = b * s
    qkv = round_to_bf16(rng.standard_normal((M, 3 * h)).astype(np.float32))
    d_attn = round_to_bf16(rng.standard_normal((M, h)).astype(np.float32))
    attn_o, _ = oatt.forward(qkv, b, s, n, causal, keep_probs=False)
    lse_o = oatt.logsumexp(qkv, b, s, n, causal)
    dqkv_o = oatt.backward(qkv, d_attn, b, s, n, causal)

    nmat = (b // q) * (n // q)
    dQKV = mat_to_dev(qkv, q, "bf16")
    O = empty(M * h, "bf16")
    L = empty(q * q * nmat * s, "fp32")
    print(f"fused attention b={b} s={s} h={n}x{h // n} q={q} causal={causal}", flush=True)
    opt.attention_fused_fwd(dQKV, O, L, b, s, h, n, q, -1, -1, causal, opt.BF16)
    torch.cuda.synchronize()
    assert rel_frobenius(mat_to_host(O, M, h, q), attn_o) <= TOL
    got_l = to_host(L).reshape(q, q, nmat, s)
    assert rel_frobenius(got_l, _lse_blocks(lse_o, b, n, q)) <= TOL_LSE

    nbytes = opt.attention_fused_workspace_bytes(b, s, h, n, q)
    assert nbytes >= q * q * nmat * s * 4
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    dO = mat_to_dev(d_attn, q, "bf16")
    dQ = empty(M * 3 * h, "bf16")
    opt.attention_fused_bwd(dQKV, O, L, dO, dQ, b, s, h, n, q, -1, -1, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    got = mat_to_host(dQ, M, 3 * h, q)
    assert rel_frobenius(got, dqkv_o) <= TOL
    d = h // n
    cols = np.arange(3 * h)
    for part in range(3):   # Q, K, V gradients separately, so a weak one cannot hide behind a strong one
        sel = (cols // d) % 3 == part
        assert rel_frobenius(got[:, sel], dqkv_o[:, sel]) <= TOL, part

    # one device only: same bits for its blocks, nothing else written
    i, j = q - 1, 0
    O1, L1, dQ1 = empty(M * h, "bf16"), empty(q * q * nmat * s, "fp32"), empty(M * 3 * h, "bf16")
    opt.attention_fused_fwd(dQKV, O1, L1, b, s, h, n, q, i, j, causal, opt.BF16)
    opt.attention_fused_bwd(dQKV, O, L, dO, dQ1, b, s, h, n, q, i, j, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    dev = i * q + j
    for full, one, blk in ((O, O1, (M // q) * (h // q)), (L, L1, nmat * s), (dQ, dQ1, (M // q) * (3 * h // q))):
        a, a1 = to_host(full), to_host(one)
        sl = slice(dev * blk, (dev + 1) * blk)
        assert np.array_equal(a[sl], a1[sl])
        mask = np.ones(a.size, dtype=bool)
        mask[sl] = False
        assert np.all(np.isnan(a1[mask]))


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("s", [1, 2, 31, 63, 64, 65, 127, 128, 129, 191, 193])
def test_fused_attention_block_boundaries(s, causal):
    """Sequence lengths around the 32-row wavefront tiles, the 64-row blocks and the 128-row load pairs (forward and
    backward, one (sequence, head) pair per device, head width 64)."""
    b, h, n, q = 2, 128, 2, 2
    rng = np.random.default_rng(s)
    M = b * s
    qkv = round_to_bf16(rng.standard_normal((M, 3 * h)).astype(np.float32))
    d_attn = round_to_bf16(rng.standard_normal((M, h)).astype(np.float32))
    attn_o, _ = oatt.forward(qkv, b, s, n, causal, keep_probs=False)
    lse_o = oatt.logsumexp(qkv, b, s, n, causal)
    dqkv_o = oatt.backward(qkv, d_attn, b, s, n, causal)
    dQKV, dO = mat_to_dev(qkv, q, "bf16"), mat_to_dev(d_attn, q, "bf16")
    O, L, dQ = empty(M * h, "bf16"), empty(q * q * s, "fp32"), empty(M * 3 * h, "bf16")
    ws = torch.empty(max(256, opt.attention_fused_workspace_bytes(b, s, h, n, q)), dtype=torch.uint8, device="cuda:0")
    opt.attention_fused_fwd(dQKV, O, L, b, s, h, n, q, -1, -1, causal, opt.BF16)
    opt.attention_fused_bwd(dQKV, O, L, dO, dQ, b, s, h, n, q, -1, -1, causal, opt.BF16, ws)
    torch.cuda.synchronize()
    assert rel_frobenius(mat_to_host(O, M, h, q), attn_o) <= TOL
    assert rel_frobenius(to_host(L).reshape(q, q, 1, s), _lse_blocks(lse_o, b, n, q)) <= TOL_LSE
    got = mat_to_host(dQ, M, 3 * h, q)
    assert not np.any(np.isnan(got))
    assert rel_frobenius(got, dqkv_o) <= TOL


@pytest.mark.parametrize("b,s,h,n,q,dev", [(8, 1024, 4096, 32, 4, (1, 2)), (64, 512, 4096, 32, 8, (6, 3)), (8, 512, 1024, 16, 4, (3, 1))],
                         ids=["config4", "config5", "config2"])
def test_fused_attention_at_benchmark_sizes(b, s, h, n, q, dev):
    """Configs 4, 5 and 2 at full size, device mode as bench.py launches it: sampled (sequence, head) pairs of the
    device recomputed by the oracle from the device's own inputs; device mode = grid mode bit for bit."""
    d = h // n
    M, nb, nh = b * s, b // q, n // q
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(s + q)
    qkv = (torch.randn(M * 3 * h, generator=gen, device="cuda:0") * 0.7).to(torch.bfloat16)      # block-major
    d_attn = torch.randn(M * h, generator=gen, device="cuda:0").to(torch.bfloat16)
    nmat = nb * nh
    i, j = dev
    O, L, dQ = empty(M * h, "bf16"), empty(q * q * nmat * s, "fp32"), empty(M * 3 * h, "bf16")
    ws = torch.empty(opt.attention_fused_workspace_bytes(b, s, h, n, q), dtype=torch.uint8, device="cuda:0")
    opt.attention_fused_fwd(qkv, O, L, b, s, h, n, q, i, j, True, opt.BF16)
    opt.attention_fused_bwd(qkv, O, L, d_attn, dQ, b, s, h, n, q, i, j, True, opt.BF16, ws)
    torch.cuda.synchronize()
    dev_id = i * q + j
    qb = qkv.view(q * q, nb * s, 3 * h // q)[dev_id]
    ob, gb, dqb = (t.view(q * q, nb * s, -1)[dev_id] for t in (O, d_attn, dQ))
    lb = L.view(q * q, nmat, s)[dev_id]
    rng = np.random.default_rng(0)
    for _ in range(3):
        seq, head = int(rng.integers(nb)), int(rng.integers(nh))
        rows = slice(seq * s, (seq + 1) * s)
        blk = to_host(qb[rows, head * 3 * d:(head + 1) * 3 * d].reshape(-1)).reshape(s, 3 * d).astype(np.float64)
        Qh, Kh, Vh = blk[:, :d], blk[:, d:2 * d], blk[:, 2 * d:]
        O_o, P_o = oatt.head_forward(Qh, Kh, Vh, True)
        assert rel_frobenius(to_host(ob[rows, head * d:(head + 1) * d].reshape(-1)).reshape(s, d), O_o) <= TOL
        assert rel_frobenius(to_host(lb[seq * nh + head]), oatt.head_logsumexp(Qh, Kh, True)) <= TOL_LSE
        dO = to_host(gb[rows, head * d:(head + 1) * d].reshape(-1)).reshape(s, d).astype(np.float64)
        want = np.concatenate(oatt.head_backward(Qh, Kh, Vh, P_o, dO), axis=1)
        got = to_host(dqb[rows, head * 3 * d:(head + 1) * 3 * d].reshape(-1)).reshape(s, 3 * d)
        assert rel_frobenius(got, want) <= TOL
    # grid mode writes the same bits into this device's blocks
    O2, L2, dQ2 = empty(M * h, "bf16"), empty(q * q * nmat * s, "fp32"), empty(M * 3 * h, "bf16")
    opt.attention_fused_fwd(qkv, O2, L2, b, s, h, n, q, -1, -1, True, opt.BF16)
    opt.attention_fused_bwd(qkv, O2, L2, d_attn, dQ2, b, s, h, n, q, -1, -1, True, opt.BF16, ws)
    torch.cuda.synchronize()
    for a_, b_ in ((O, O2), (dQ, dQ2)):
        assert torch.equal(a_.view(q * q, -1)[dev_id].view(torch.int16), b_.view(q * q, -1)[dev_id].view(torch.int16))
    assert torch.equal(L.view(q * q, -1)[dev_id].view(torch.int32), L2.view(q * q, -1)[dev_id].view(torch.int32))


def test_fused_attention_closed_forms():
    """Q = 0: uniform weights over the visible prefix, O_t = mean(V_0..t) and L_t = log(t + 1)."""
    b, s, h, n, q = 2, 200, 128, 2, 1
    d = h // n
    rng = np.random.default_rng(3)
    qkv = rng.standard_normal((b * s, 3 * h)).astype(np.float32)
    cols = np.arange(3 * h)
    qkv[:, (cols // d) % 3 == 0] = 0.0
    qkv = round_to_bf16(qkv)
    O, L = empty(b * s * h, "bf16"), empty(b * n * s, "fp32")
    opt.attention_fused_fwd(mat_to_dev(qkv, q, "bf16"), O, L, b, s, h, n, q, 0, 0, True, opt.BF16)
    torch.cuda.synchronize()
    out = mat_to_host(O, b * s, h, q)
    for seq in range(b):
        for head in range(n):
            V = qkv[seq * s:(seq + 1) * s, head * 3 * d + 2 * d:head * 3 * d + 3 * d].astype(np.float64)
            want = np.cumsum(V, axis=0) / np.arange(1, s + 1)[:, None]
            assert rel_frobenius(out[seq * s:(seq + 1) * s, head * d:(head + 1) * d], want) <= TOL
    assert np.allclose(to_host(L).reshape(b * n, s), np.log(np.arange(1, s + 1))[None, :], atol=1e-5)


def test_fused_attention_errors():
    one = empty(16, "bf16")
    lse = empty(16, "fp32")
    for args, code in [((3, 64, 128, 2, 2), opt.ESHAPE),     # b not divisible by q
                       ((4, 64, 128, 3, 2), opt.ESHAPE),     # n not divisible by q
                       ((4, 64, 64, 4, 2), opt.ESHAPE)]:     # head width 16: not built
        with pytest.raises(opt.OptimusError) as e:
            opt.attention_fused_fwd(one, one, lse, *args, 0, 0, True, opt.BF16)
        assert e.value.code == code
    with pytest.raises(opt.OptimusError) as e:
        opt.attention_fused_bwd(one, one, lse, one, one, 4, 64, 128, 2, 2, 0, 0, True, opt.BF16, None)
    assert e.value.code == opt.EWORKSPACE
