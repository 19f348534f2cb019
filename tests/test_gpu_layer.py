"""GPU parity: one transformer layer (forward and backward) on the q x q grid against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import layer as olayer
from oracle.metrics import rel_frobenius
from workloads import LayerShape, layer_inputs, CONFIGS
from gpu_util import to_host
from layer_util import (alloc_layer, fetch, compare_all, TOL, FWD_OUT, BWD_OUT, FP32_MATS, MAT_SHAPES)

pytestmark = pytest.mark.gpu
# Every comparison below is against the exact oracle (fp64, nothing rounded anywhere).  Bounds per tensor:
# layer_util.bound -- 5e-3, and the stated wider bound for the gradients behind the soft-max logits.


def _oracle(inp, shp, causal, keep_probs=True):
    fe = olayer.forward(inp, shp.b, shp.s, shp.n, causal=causal, keep_probs=keep_probs)
    be = olayer.backward(inp, fe, shp.b, shp.s, shp.n, causal=causal)
    return fe, be


def _scale_weights(inp, shp):
    """Weights larger than the benchmark recipe's N(0, 0.02^2), which at these small h would leave the attention
    and MLP branches without signal: scaled so that a projection of an N(0,1) row has standard deviation 0.9
    whatever h (soft-max logits of standard deviation about 0.8; the full-size tests cover the benchmark
    layers' own scale, 1.6)."""
    from workloads import round_to_bf16
    f = 4.0 * (128.0 / shp.h) ** 0.5
    for k in ("w_qkv", "w_o", "w1", "w2"):
        inp[k] = round_to_bf16(inp[k] * f)


def _fmt(w):
    return {k: f"{v:.2e}" for k, v in w.items()}


# several tiles + ragged sizes (h/q = 72 is not a tile multiple), q = 1 (no partition), q = 2, 4
SMALL = [LayerShape(b=4, s=64, h=128, n=4, q=2), LayerShape(b=2, s=136, h=144, n=2, q=2),
         LayerShape(b=2, s=128, h=256, n=4, q=1), LayerShape(b=4, s=72, h=256, n=8, q=4)]


@pytest.mark.parametrize("shp", SMALL, ids=lambda s: f"b{s.b}s{s.s}h{s.h}n{s.n}q{s.q}")
@pytest.mark.parametrize("causal", [True, False])
def test_layer_grid_and_device_mode(shp, causal):
    inp = layer_inputs(11, shp, "bf16", perturb_affine=True)
    _scale_weights(inp, shp)
    fe, be = _oracle(inp, shp, causal)
    cfg, T, lt, ws = alloc_layer(inp, shp, causal)
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    w_e = compare_all(T, shp, inp, fe, be)
    print("vs exact oracle:", _fmt(w_e))

    # device mode: recompute one device's blocks from the resident peers; bits must not change anywhere
    snap = {k: v.clone() for k, v in T.items()}
    i, j = shp.q - 1, 0
    opt.layer_fwd(cfg, lt, i, j, ws)
    opt.layer_bwd(cfg, lt, i, j, ws)
    torch.cuda.synchronize()
    for k, v in T.items():
        a, b = v.view(torch.int16 if v.dtype == torch.bfloat16 else torch.int32), snap[k].view(torch.int16 if v.dtype == torch.bfloat16 else torch.int32)
        assert torch.equal(a, b), f"{k} changed between grid mode and device mode"


# head widths 64 and 128 (what the attention without [s x s] tensors is built for), ragged s, q = 1, 2
FUSED = [LayerShape(b=4, s=72, h=256, n=4, q=2), LayerShape(b=2, s=136, h=256, n=2, q=2),
         LayerShape(b=2, s=128, h=128, n=2, q=1)]


@pytest.mark.parametrize("shp", FUSED, ids=lambda s: f"b{s.b}s{s.s}h{s.h}n{s.n}q{s.q}")
@pytest.mark.parametrize("causal", [True, False])
def test_layer_with_fused_attention(shp, causal):
    """The layer with cfg.fused_attention = 1: same oracles, same tolerances; no probs tensor, lse instead."""
    from oracle import attention as oatt
    from workloads import round_to_bf16
    inp = layer_inputs(13, shp, "bf16", perturb_affine=True)
    _scale_weights(inp, shp)
    fe, be = _oracle(inp, shp, causal)
    cfg, T, lt, ws = alloc_layer(inp, shp, causal, fused=True)
    assert "probs" not in T and cfg.fused_attention == 1
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    w_e = compare_all(T, shp, inp, fe, be)
    print("fused, vs exact oracle:", _fmt(w_e))
    # the attention stage by itself, from the values the device stored for its inputs, to the per-stage tolerance
    qkv_dev = fetch(T, "qkv", shp)
    attn_o, _ = oatt.forward(qkv_dev, shp.b, shp.s, shp.n, causal, keep_probs=False)
    assert rel_frobenius(fetch(T, "attn", shp), attn_o) <= TOL
    dqkv_o = oatt.backward(qkv_dev, fetch(T, "d_attn", shp), shp.b, shp.s, shp.n, causal)
    assert rel_frobenius(fetch(T, "d_qkv", shp), dqkv_o) <= TOL
    # the saved row statistic, against the oracle's log-sum-exp of the qkv the device stored
    q, nb, nh = shp.q, shp.b // shp.q, shp.n // shp.q
    L = oatt.logsumexp(qkv_dev, shp.b, shp.s, shp.n, causal)
    got = to_host(T["lse"]).reshape(q, q, nb * nh, shp.s)
    for i in range(q):
        for j in range(q):
            want = L[i * nb:(i + 1) * nb, j * nh:(j + 1) * nh].reshape(nb * nh, shp.s)
            assert rel_frobenius(got[i, j], want) <= 1e-5
    snap = {k: v.clone() for k, v in T.items()}
    i, j = shp.q - 1, 0
    opt.layer_fwd(cfg, lt, i, j, ws)
    opt.layer_bwd(cfg, lt, i, j, ws)
    torch.cuda.synchronize()
    for k, v in T.items():
        assert torch.equal(v.view(torch.uint8), snap[k].view(torch.uint8)), f"{k} changed between grid mode and device mode"


def test_layer_fused_attention_rejects_other_head_widths():
    shp = LayerShape(b=4, s=64, h=128, n=4, q=2)   # h/n = 32
    cfg = opt.LayerCfg(shp.b, shp.s, shp.h, shp.n, shp.q, 1e-5, 1, opt.BF16, 1)
    assert opt.layer_workspace_bytes(cfg) == 0
    with pytest.raises(opt.OptimusError) as e:
        opt.layer_fwd(cfg, opt.make_layer_tensors({}), 0, 0, None)
    assert e.value.code == opt.ESHAPE


def test_layer_device_mode_writes_only_its_blocks():
    shp = LayerShape(b=4, s=64, h=128, n=4, q=2)
    inp = layer_inputs(12, shp, "bf16", perturb_affine=True)
    cfg, T, lt, ws = alloc_layer(inp, shp, True)
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    ref = {k: to_host(v).copy() for k, v in T.items()}
    outs = [k for k in T if k in FWD_OUT + BWD_OUT + FP32_MATS]
    # every stage reads the peers' resident blocks, so the write set is checked this way: overwrite device
    # (1,0)'s blocks with NaN, rerun device (1,0) only, and everything must equal the grid result again
    i, j, q = 1, 0, shp.q
    for k in outs:
        r, c = MAT_SHAPES[k](shp.M, shp.h)
        blk = (r // q) * (c // q)
        T[k][(i * q + j) * blk:(i * q + j + 1) * blk] = float("nan")
    opt.layer_fwd(cfg, lt, i, j, ws)
    opt.layer_bwd(cfg, lt, i, j, ws)
    torch.cuda.synchronize()
    for k in outs:
        assert np.array_equal(to_host(T[k]), ref[k]), k


def test_layer_config2_full_size():
    """Benchmark configuration 2 (b=8, s=512, h=1024, 16 heads, q=4) at full size: grid run vs the oracle,
    then the timed launch configuration (one device, resident peers) reproduces its blocks bit for bit."""
    shp = CONFIGS["config2"]["layer"]
    inp = layer_inputs(CONFIGS["config2"]["seed"], shp, "bf16")
    fe, be = _oracle(inp, shp, True, keep_probs=False)
    cfg, T, lt, ws = alloc_layer(inp, shp, True)
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    w_e = compare_all(T, shp, inp, fe, be)
    print("config2 full size, vs exact oracle:", _fmt(w_e))
    snap = {k: v.clone() for k, v in T.items()}
    opt.layer_fwd(cfg, lt, 3, 1, ws)
    opt.layer_bwd(cfg, lt, 3, 1, ws)
    torch.cuda.synchronize()
    for k, v in T.items():
        assert torch.equal(v.view(torch.uint8), snap[k].view(torch.uint8)), k
    # the benchmark replays the step of device (1, 2) from a HIP graph: every replay, with eager work and
    # synchronisations in between, must leave the grid run's bits (its blocks are poisoned before each replay)
    outs = [k for k in T if k in FWD_OUT + BWD_OUT + FP32_MATS]
    i, j, q = 1, 2, shp.q

    def step():
        opt.layer_fwd(cfg, lt, i, j, ws)
        opt.layer_bwd(cfg, lt, i, j, ws)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for replay in range(3):
        for k in outs:
            r, c = MAT_SHAPES[k](shp.M, shp.h)
            blk = (r // q) * (c // q)
            T[k][(i * q + j) * blk:(i * q + j + 1) * blk] = float("nan")
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k, v in T.items():
            assert torch.equal(v.view(torch.uint8), snap[k].view(torch.uint8)), (replay, k)
        opt.layer_fwd(cfg, lt, 0, 3, ws)   # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("shp", [LayerShape(b=4, s=64, h=128, n=4, q=2), LayerShape(b=8, s=1024, h=2048, n=16, q=2),
                                 LayerShape(b=8, s=512, h=1024, n=16, q=4)],
                         ids=["small_blocks", "large_blocks", "config2_panel_split"])
def test_layer_layernorm_parameter_gradients_equal_the_standalone_call(shp):
    """The layer runs the LayerNorm parameter gradients on either of its two streams depending on the block size
    ([128 x 64]: the gradient branch; [4096 x 1024]: the activation chain).  Wherever they run, they are the column
    sums of the stored dY and dY * xhat: bit-identical to optimus_layernorm2d_bwd on the same stored tensors."""
    inp = layer_inputs(14, shp, "bf16", perturb_affine=True)
    cfg, T, lt, ws = alloc_layer(inp, shp, True)
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    M, h, q = shp.M, shp.h, shp.q
    for k, dy, res in (("2", "d_ln2_out", "d_out"), ("1", "d_ln1_out", "d_h_mid")):
        dg, db = torch.full_like(T["d_ln%s_g" % k], float("nan")), torch.full_like(T["d_ln%s_b" % k], float("nan"))
        dx = torch.empty_like(T[dy])
        stats = torch.empty_like(T["bstats" + k])
        opt.layernorm2d_bwd(T[dy], T["xhat" + k], T["rstd" + k], T["ln%s_g" % k], T[res], dx, dg, db, stats, M, h, q, -1, -1, opt.BF16)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(dg), to_host(T["d_ln%s_g" % k])), k
        assert np.array_equal(to_host(db), to_host(T["d_ln%s_b" % k])), k
        assert np.array_equal(to_host(dx), to_host(T["d_h_mid" if k == "2" else "d_x"])), k
    # The dY the two LayerNorm backward kernels read is the layer's own product (planned as one of two products that
    # run side by side, panel-split at config 2): it has the bits of the standalone product on the same stored
    # operands, and a single device's backward pass reproduces the grid run's bits.
    for dy, a_name, w_name, K in (("d_ln2_out", "d_pre_gelu", "w1", 4 * h), ("d_ln1_out", "d_qkv", "w_qkv", 3 * h)):
        nbytes = max(opt.summa_workspace_bytes("abt", M, K, h, q, -1, -1, opt.BF16), opt.summa_workspace_bytes("abt", M, K, h, q, 0, 0, opt.BF16))
        ws2 = torch.empty(max(256, nbytes), dtype=torch.uint8, device="cuda:0")
        Cm = torch.empty_like(T[dy])
        opt.summa("abt", T[a_name], T[w_name], Cm, M, K, h, q, -1, -1, opt.BF16, ws=ws2)
        torch.cuda.synchronize()
        print(dy, "standalone plan (variant, splits):", opt.binding.debug_last_gemm_plan())
        assert torch.equal(Cm.view(torch.int16), T[dy].view(torch.int16)), dy
    snap = {k_: v.clone() for k_, v in T.items()}
    i, j = q - 1, 0
    for k_ in ("d_ln2_out", "d_ln1_out", "d_h_mid", "d_x"):
        blk = (M // q) * (h // q)
        T[k_][(i * q + j) * blk:(i * q + j + 1) * blk] = float("nan")
    opt.layer_bwd(cfg, lt, i, j, ws)
    torch.cuda.synchronize()
    for k_, v in T.items():
        assert torch.equal(v.view(torch.uint8), snap[k_].view(torch.uint8)), k_


def test_layer_errors():
    shp = LayerShape(b=4, s=64, h=128, n=4, q=2)
    inp = layer_inputs(1, shp, "bf16")
    cfg, T, lt, ws = alloc_layer(inp, shp, True)
    small = torch.empty(64, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(opt.OptimusError) as e:
        opt.layer_fwd(cfg, lt, -1, -1, small)
    assert e.value.code == opt.EWORKSPACE
    with pytest.raises(opt.OptimusError) as e:
        opt.layer_fwd(cfg, lt, 0, 2, ws)
    assert e.value.code == opt.ECOORD
    bad = opt.LayerCfg(shp.b, shp.s, shp.h, 3, shp.q, 1e-5, 1, opt.BF16)
    with pytest.raises(opt.OptimusError) as e:
        opt.layer_fwd(bad, lt, -1, -1, ws)
    assert e.value.code == opt.ESHAPE
    T2 = dict(T)
    T2["w1"] = None
    with pytest.raises(opt.OptimusError) as e:
        opt.layer_fwd(cfg, opt.make_layer_tensors(T2), -1, -1, ws)
    assert e.value.code == opt.EINVAL


def test_first_call_under_graph_capture_then_eager():
    """In a fresh process the very first layer_fwd/layer_bwd calls are made while a HIP graph is being captured
    (the library must not create its gradient-branch stream there); replays, then eager calls (which do create it),
    then a second captured graph with the forked branch: all give the same bits."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r'''
import sys
sys.path.insert(0, ROOT); sys.path.insert(0, ROOT + "/tests")
import torch
import paper_2104_05343_amd as opt
from workloads import LayerShape, layer_inputs
from layer_util import alloc_layer
shp = LayerShape(b=4, s=64, h=128, n=4, q=2)
inp = layer_inputs(3, shp, "bf16", perturb_affine=True)
cfg, T, lt, ws = alloc_layer(inp, shp, True)
def step():
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
def snap():
    torch.cuda.synchronize()
    return {k: v.clone() for k, v in T.items()}
def same(a, b):
    return all(torch.equal(a[k].view(torch.uint8), b[k].view(torch.uint8)) for k in a)
side = torch.cuda.Stream()
with torch.cuda.stream(side):
    g1 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g1):
        step()
g1.replay(); r1 = snap()
g1.replay(); r2 = snap()
step(); e1 = snap()
g2 = torch.cuda.CUDAGraph()
with torch.cuda.graph(g2):
    step()
g2.replay(); r3 = snap()
step(); e2 = snap()
g2.replay(); r4 = snap()
assert same(r1, r2) and same(r1, e1) and same(r1, r3) and same(r1, e2) and same(r1, r4)
assert not any(torch.isnan(v.float()).any().item() for k, v in r1.items() if k in ("out", "d_x", "d_w1", "d_b1"))
print("capture-first ok")
'''.replace("ROOT", repr(root))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "capture-first ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
