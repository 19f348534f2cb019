"""Pins for oracle/layer.py: GeLU against math.erf, the full backward against
finite differences of <d_out, out> on a tiny layer, Table-1-style structure."""
import math

import numpy as np

from oracle import layer
from workloads import LayerShape, layer_inputs


def test_gelu_against_math_erf():
    z = np.linspace(-6, 6, 241)
    want = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in z])
    assert np.allclose(layer.gelu(z), want, atol=1e-15)
    assert layer.gelu(np.array([0.0]))[0] == 0.0
    assert abs(layer.gelu(np.array([10.0]))[0] - 10.0) < 1e-12
    hstep = 1e-6
    fd = (layer.gelu(z + hstep) - layer.gelu(z - hstep)) / (2 * hstep)
    assert np.allclose(layer.gelu_grad(z), fd, atol=1e-8)


def _loss(inp, shp):
    f = layer.forward(inp, shp.b, shp.s, shp.n, causal=True, keep_probs=False)
    return float(np.sum(np.asarray(inp["d_out"], dtype=np.float64) * f["out"]))


def test_layer_backward_finite_differences():
    shp = LayerShape(b=2, s=4, h=8, n=2, q=2)
    inp = {k: np.asarray(v, dtype=np.float64) for k, v in layer_inputs(5, shp, "fp32", perturb_affine=True).items()}
    # larger weights so that every path carries signal
    for k in ("w_qkv", "w_o", "w1", "w2"):
        inp[k] = inp[k] * 20.0
    fwd = layer.forward(inp, shp.b, shp.s, shp.n, causal=True)
    g = layer.backward(inp, fwd, shp.b, shp.s, shp.n, causal=True)
    names = {"x": "d_x", "w_qkv": "d_w_qkv", "b_qkv": "d_b_qkv", "w_o": "d_w_o", "b_o": "d_b_o",
             "w1": "d_w1", "b1": "d_b1", "w2": "d_w2", "b2": "d_b2",
             "ln1_g": "d_ln1_g", "ln1_b": "d_ln1_b", "ln2_g": "d_ln2_g", "ln2_b": "d_ln2_b"}
    rng = np.random.default_rng(0)
    hstep = 1e-5
    for name, gname in names.items():
        T = inp[name]
        idxs = list(np.ndindex(*T.shape))
        pick = [idxs[k] for k in rng.choice(len(idxs), size=min(12, len(idxs)), replace=False)]
        for idx in pick:
            old = T[idx]
            T[idx] = old + hstep
            lp = _loss(inp, shp)
            T[idx] = old - hstep
            lm = _loss(inp, shp)
            T[idx] = old
            fd = (lp - lm) / (2 * hstep)
            assert abs(fd - g[gname][idx]) < 1e-5 * max(1.0, abs(fd)), (name, idx, fd, g[gname][idx])


def test_layer_forward_structure():
    shp = LayerShape(b=2, s=4, h=8, n=2, q=2)
    inp = layer_inputs(6, shp, "fp32", perturb_affine=True)
    f = layer.forward(inp, shp.b, shp.s, shp.n)
    # zero output-projection and zero second MLP matrix -> pure residual path
    inp2 = dict(inp)
    inp2["w_o"] = np.zeros_like(inp["w_o"])
    inp2["w2"] = np.zeros_like(inp["w2"])
    f2 = layer.forward(inp2, shp.b, shp.s, shp.n)
    want = np.asarray(inp["x"], dtype=np.float64) + inp["b_o"][None, :] + inp["b2"][None, :]
    assert np.allclose(f2["out"], want, atol=1e-12)
    # causality: changing the last token of a sequence leaves earlier tokens unchanged
    inp3 = dict(inp)
    x3 = np.array(inp["x"], dtype=np.float64)
    x3[shp.s - 1] += 1.0
    inp3["x"] = x3
    f3 = layer.forward(inp3, shp.b, shp.s, shp.n)
    assert np.allclose(f3["out"][:shp.s - 1], f["out"][:shp.s - 1], atol=1e-12)
    assert not np.allclose(f3["out"][shp.s - 1], f["out"][shp.s - 1])
    # sequences are independent
    assert np.allclose(f3["out"][shp.s:], f["out"][shp.s:], atol=1e-12)
