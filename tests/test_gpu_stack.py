"""GPU parity: a stack of layers with activation checkpointing and shared, pre-allocated buffers against the fp64
oracle, and bit for bit against the same layers run one by one with every tensor kept (recomputation changes no bit)."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import stack as ostack
from oracle.metrics import rel_frobenius
from workloads import LayerShape, layer_inputs, round_to_bf16
from gpu_util import mat_to_dev, mat_to_host, to_host, vec_to_dev, empty
from layer_util import alloc_layer, MAT_SHAPES, TOL_BEHIND_LOGITS

pytestmark = pytest.mark.gpu
MATS = ("w_qkv", "w_o", "w1", "w2")
VEC_MULT = {"d_b_qkv": 3, "d_b_o": 1, "d_b1": 4, "d_b2": 1, "d_ln1_g": 1, "d_ln1_b": 1, "d_ln2_g": 1, "d_ln2_b": 1}


def _inputs(seed, shp, L):
    layers = []
    for l in range(L):
        inp = layer_inputs(seed + l, shp, "bf16", perturb_affine=True)
        for k in MATS:
            inp[k] = round_to_bf16(inp[k] * 4.0)
        layers.append(inp)
    return layers, layers[0]["x"], layers[0]["d_out"]


def _buffers(cfg, L):
    sz = opt.stack_sizes(cfg, L)
    raw = {k: torch.full((max(1, getattr(sz, k)),), 0xFF, dtype=torch.uint8, device="cuda:0")   # 0xFFFF bf16 = NaN
           for k in ("workspace", "forward", "backward", "conjunction", "checkpoint")}
    return sz, raw, opt.make_stack_buffers(raw["workspace"], raw["forward"], raw["backward"], raw["conjunction"], raw["checkpoint"])


def _alloc_grads(shp):
    h, q = shp.h, shp.q
    g = {"d_w_qkv": empty(3 * h * h, "fp32"), "d_w_o": empty(h * h, "fp32"), "d_w1": empty(4 * h * h, "fp32"),
         "d_w2": empty(4 * h * h, "fp32")}
    for k, m in VEC_MULT.items():
        g[k] = empty(q * m * h, "fp32")
    return g


@pytest.mark.parametrize("shp,L,fused", [(LayerShape(b=4, s=64, h=128, n=4, q=2), 3, False),
                                        (LayerShape(b=2, s=72, h=256, n=4, q=2), 2, True),
                                        (LayerShape(b=2, s=64, h=128, n=2, q=1), 2, False)],
                         ids=["q2-L3", "q2-L2-fused", "q1-L2"])
def test_stack_against_oracle_and_layerwise_run(shp, L, fused):
    M, h, q = shp.M, shp.h, shp.q
    layers, x, d_out = _inputs(21, shp, L)
    params_o = [{k: inp[k] for k in ostack.PARAM_NAMES} for inp in layers]
    out_o, ck_o = ostack.forward(params_o, x, shp.b, shp.s, shp.n, True)
    dx_o, grads_o = ostack.backward(params_o, ck_o, d_out, shp.b, shp.s, shp.n, True)
    # Against the exact oracle (nothing rounded).  One layer's deepest gradients are held to TOL_BEHIND_LOGITS (tests
    # of the layer); in a stack the input gradient and the first layer's parameter gradients have passed through all
    # L layers forward and back, each adding its own independent rounding error, so the bound grows with the
    # number of layer passes behind a tensor: TOL_BEHIND_LOGITS * sqrt(2 L).  The sharper statement is the bit-for-bit
    # comparison with the layer-by-layer run below, whose every layer is covered by the layer tests.
    tol = TOL_BEHIND_LOGITS * float(np.sqrt(2 * L))

    cfg = opt.LayerCfg(shp.b, shp.s, shp.h, shp.n, shp.q, 1e-5, 1, opt.BF16, 1 if fused else 0)
    dev_params = []
    for inp in layers:
        t = {k: mat_to_dev(inp[k], q, "bf16") for k in MATS}
        t.update({k: vec_to_dev(inp[k]) for k in ostack.PARAM_NAMES if k not in MATS})
        dev_params.append(t)
    P = [opt.make_layer_params(t) for t in dev_params]
    sz, raw, buf = _buffers(cfg, L)
    X, dO = mat_to_dev(x, q, "bf16"), mat_to_dev(d_out, q, "bf16")
    OUT, dX = empty(M * h, "bf16"), empty(M * h, "bf16")
    G = [_alloc_grads(shp) for _ in range(L)]
    print(f"stack L={L} fused={fused} sizes", {k: getattr(sz, k) for k, _ in sz._fields_}, flush=True)
    opt.stack_fwd(cfg, P, X, buf, OUT)
    opt.stack_bwd(cfg, P, [opt.make_layer_grads(g) for g in G], dO, buf, dX)
    torch.cuda.synchronize()

    worst = {"out": rel_frobenius(mat_to_host(OUT, M, h, q), out_o), "d_x": rel_frobenius(mat_to_host(dX, M, h, q), dx_o)}
    ck = raw["checkpoint"].view(torch.bfloat16)
    for l in range(L):
        worst[f"ck{l}"] = rel_frobenius(mat_to_host(ck[l * M * h:(l + 1) * M * h], M, h, q), ck_o[l])
        for k in MATS:
            r, c = MAT_SHAPES["d_" + k](M, h)
            worst[f"L{l}.d_{k}"] = rel_frobenius(mat_to_host(G[l]["d_" + k], r, c, q), grads_o[l]["d_" + k])
        for k in VEC_MULT:   # per-device partials [q][q][N/q]: summed over the grid rows they are the gradient
            got = to_host(G[l][k]).reshape(q, q, -1).sum(axis=0).reshape(-1)
            worst[f"L{l}.{k}"] = rel_frobenius(got, grads_o[l][k])
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"over tolerance {tol}: {bad}\nall: {worst}"
    print("stack worst error %.2e (bound %.2e)" % (max(worst.values()), tol), {k: f"{v:.1e}" for k, v in worst.items()})

    # the same layers one by one, every tensor kept, no recomputation: the stack must reproduce these bits
    cur = X
    kept = []
    for l in range(L):
        inp = dict(layers[l])
        cfg_l, T, lt, ws = alloc_layer(inp, shp, True, fused=fused)
        T["x"].copy_(cur)
        lt = opt.make_layer_tensors(T)
        opt.layer_fwd(cfg_l, lt, -1, -1, ws)
        kept.append((cfg_l, T, ws))
        cur = T["out"]
    torch.cuda.synchronize()
    assert torch.equal(cur.view(torch.int16), OUT.view(torch.int16))
    g_in = dO
    for l in range(L - 1, -1, -1):
        cfg_l, T, ws = kept[l]
        T["d_out"].copy_(g_in)
        opt.layer_bwd(cfg_l, opt.make_layer_tensors(T), -1, -1, ws)
        torch.cuda.synchronize()
        for k in list(VEC_MULT) + ["d_" + m for m in MATS]:
            assert torch.equal(T[k].view(torch.int32), G[l][k].view(torch.int32)), (l, k)
        g_in = T["d_x"]
    assert torch.equal(g_in.view(torch.int16), dX.view(torch.int16))


def test_stack_graph_replays_equal_eager():
    """The benchmark times the stack from a HIP graph (a device-to-device copy node, the recomputation and the forked
    gradient branch of every layer).  Every replay, with eager work and synchronisations between them and the outputs
    poisoned before each, leaves the bits of the eager run."""
    shp, L = LayerShape(b=4, s=64, h=128, n=4, q=2), 3
    M, h, q = shp.M, shp.h, shp.q
    layers, x, d_out = _inputs(31, shp, L)
    cfg = opt.LayerCfg(shp.b, shp.s, shp.h, shp.n, shp.q, 1e-5, 1, opt.BF16, 0)
    dev_params = []
    for inp in layers:
        t = {k: mat_to_dev(inp[k], q, "bf16") for k in MATS}
        t.update({k: vec_to_dev(inp[k]) for k in ostack.PARAM_NAMES if k not in MATS})
        dev_params.append(t)
    P = [opt.make_layer_params(t) for t in dev_params]
    sz, raw, buf = _buffers(cfg, L)
    X, dO = mat_to_dev(x, q, "bf16"), mat_to_dev(d_out, q, "bf16")
    OUT, dX = empty(M * h, "bf16"), empty(M * h, "bf16")
    G = [_alloc_grads(shp) for _ in range(L)]
    GL = [opt.make_layer_grads(g) for g in G]

    def step():
        opt.stack_fwd(cfg, P, X, buf, OUT)
        opt.stack_bwd(cfg, P, GL, dO, buf, dX)

    def results():
        torch.cuda.synchronize()
        r = {"out": OUT.clone(), "d_x": dX.clone()}
        for l in range(L):
            r.update({f"L{l}.{k}": v.clone() for k, v in G[l].items()})
        return r

    def poison():
        OUT.view(torch.int16).fill_(-1)
        dX.view(torch.int16).fill_(-1)
        for g in G:
            for v in g.values():
                v.fill_(float("nan"))
        torch.cuda.synchronize()

    step()
    want = results()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        poison()
        graph.replay()
        got = results()
        for k in want:
            assert torch.equal(got[k].view(torch.uint8), want[k].view(torch.uint8)), (replay, k)
        opt.stack_fwd(cfg, P, X, buf, OUT)   # eager work between the replays
        torch.cuda.synchronize()


def test_stack_shared_gradient_buffer_with_callback():
    """All layers write their parameter gradients into ONE buffer; the per-layer callback takes them out (here: a
    stream-ordered copy), as an optimizer that updates a layer right after its backward pass would."""
    shp, L = LayerShape(b=4, s=64, h=128, n=4, q=2), 3
    M, h, q = shp.M, shp.h, shp.q
    layers, x, d_out = _inputs(33, shp, L)
    cfg = opt.LayerCfg(shp.b, shp.s, shp.h, shp.n, shp.q, 1e-5, 1, opt.BF16)
    dev_params = []
    for inp in layers:
        t = {k: mat_to_dev(inp[k], q, "bf16") for k in MATS}
        t.update({k: vec_to_dev(inp[k]) for k in ostack.PARAM_NAMES if k not in MATS})
        dev_params.append(t)
    P = [opt.make_layer_params(t) for t in dev_params]
    sz, raw, buf = _buffers(cfg, L)
    X, dO = mat_to_dev(x, q, "bf16"), mat_to_dev(d_out, q, "bf16")
    OUT, dX, dX2 = empty(M * h, "bf16"), empty(M * h, "bf16"), empty(M * h, "bf16")
    # reference: separate gradient tensors per layer
    G = [_alloc_grads(shp) for _ in range(L)]
    opt.stack_fwd(cfg, P, X, buf, OUT)
    opt.stack_bwd(cfg, P, [opt.make_layer_grads(g) for g in G], dO, buf, dX)
    torch.cuda.synchronize()
    shared = torch.full((sz.param_grad,), 0xFF, dtype=torch.uint8, device="cuda:0")
    lg = opt.layer_grads_in(cfg, shared)
    taken, order = {}, []

    def done(layer):
        order.append(layer)
        taken[layer] = shared.clone()     # enqueued on the same (default) stream: after this layer, before the next
    opt.stack_bwd(cfg, P, [lg] * L, dO, buf, dX2, done=done)
    torch.cuda.synchronize()
    assert order == list(range(L - 1, -1, -1))
    assert torch.equal(dX.view(torch.int16), dX2.view(torch.int16))
    base = shared.data_ptr()
    for l in range(L):
        for k in opt.binding.LAYER_GRAD_FIELDS:
            off = getattr(lg, k) - base
            n = G[l][k].numel() * 4
            assert torch.equal(taken[l][off:off + n], G[l][k].view(torch.uint8)), (l, k)


def test_stack_errors():
    cfg = opt.LayerCfg(4, 64, 128, 4, 2, 1e-5, 1, opt.BF16)
    with pytest.raises(opt.OptimusError) as e:
        opt.stack_sizes(cfg, 0)
    assert e.value.code == opt.ESHAPE
    bad = opt.LayerCfg(3, 64, 128, 4, 2, 1e-5, 1, opt.BF16)
    with pytest.raises(opt.OptimusError) as e:
        opt.stack_sizes(bad, 2)
    assert e.value.code == opt.ESHAPE
