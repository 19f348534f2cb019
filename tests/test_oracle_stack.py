"""Pins for oracle/stack.py: one layer reduces to the layer oracle, checkpoints are the layer inputs, the
gradients through two layers against central finite differences, and the count of forward passes behind the
backward rows of Table 1 (backward with checkpointing = three times the forward computation)."""
import numpy as np

from oracle import layer, stack
from workloads import LayerShape, layer_inputs


def _params(seed, shp, L, scale=20.0):
    out = []
    for l in range(L):
        inp = {k: np.asarray(v, dtype=np.float64) for k, v in layer_inputs(seed + l, shp, "fp32", perturb_affine=True).items()}
        for k in ("w_qkv", "w_o", "w1", "w2"):
            inp[k] = inp[k] * scale
        out.append({k: inp[k] for k in stack.PARAM_NAMES})
    return out


def test_one_layer_is_the_layer_oracle():
    shp = LayerShape(b=2, s=4, h=8, n=2, q=2)
    inp = {k: np.asarray(v, dtype=np.float64) for k, v in layer_inputs(3, shp, "fp32", perturb_affine=True).items()}
    p = [{k: inp[k] for k in stack.PARAM_NAMES}]
    out, ck = stack.forward(p, inp["x"], shp.b, shp.s, shp.n)
    f = layer.forward(inp, shp.b, shp.s, shp.n)
    g = layer.backward(inp, f, shp.b, shp.s, shp.n)
    assert np.array_equal(out, f["out"]) and len(ck) == 1 and np.array_equal(ck[0], inp["x"])
    dx, grads = stack.backward(p, ck, inp["d_out"], shp.b, shp.s, shp.n)
    assert np.array_equal(dx, g["d_x"])
    for k in stack.GRAD_NAMES:
        assert np.array_equal(grads[0][k], g[k]), k


def test_checkpoints_are_layer_inputs_and_forward_count():
    shp = LayerShape(b=2, s=4, h=8, n=2, q=2)
    L = 3
    p = _params(7, shp, L, scale=5.0)
    x = np.asarray(layer_inputs(1, shp, "fp32")["x"], dtype=np.float64)
    cnt = {}
    out, ck = stack.forward(p, x, shp.b, shp.s, shp.n, counter=cnt)
    assert cnt["forward_passes"] == L
    cur = x
    for l in range(L):
        assert np.array_equal(ck[l], cur)
        cur = layer.forward(dict(p[l], x=cur), shp.b, shp.s, shp.n)["out"]
    assert np.array_equal(out, cur)
    stack.backward(p, ck, np.ones_like(out), shp.b, shp.s, shp.n, counter=cnt)
    # forward 1x, backward = recomputed forward 1x + gradients 2x: Table 1's 36 = 3 * 12 and 6 = 3 * 2
    assert cnt["forward_passes"] == 2 * L


def test_two_layer_gradients_finite_differences():
    shp = LayerShape(b=2, s=3, h=8, n=2, q=1)
    p = _params(11, shp, 2)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((shp.b * shp.s, shp.h))
    R = rng.standard_normal((shp.b * shp.s, shp.h))

    def loss():
        return float(np.sum(R * stack.forward(p, x, shp.b, shp.s, shp.n)[0]))
    out, ck = stack.forward(p, x, shp.b, shp.s, shp.n)
    dx, grads = stack.backward(p, ck, R, shp.b, shp.s, shp.n)
    hstep = 1e-5
    targets = [(x, dx)] + [(p[l][k], grads[l]["d_" + k]) for l in range(2) for k in ("w_qkv", "b_o", "ln2_g", "w2", "b1")]
    for T, G in targets:
        idxs = list(np.ndindex(*T.shape))
        for idx in [idxs[k] for k in rng.choice(len(idxs), size=min(6, len(idxs)), replace=False)]:
            old = T[idx]
            T[idx] = old + hstep
            lp = loss()
            T[idx] = old - hstep
            lm = loss()
            T[idx] = old
            fd = (lp - lm) / (2 * hstep)
            assert abs(fd - G[idx]) < 2e-5 * max(1.0, abs(fd)), (idx, fd, G[idx])
