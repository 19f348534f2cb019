"""A stack of identical transformer layers run with distributed activation checkpointing
(Section 3.2.3 "memory pre-allocation and checkpointing", the figure on checkpointing, and the
backward rows of Table 1: with checkpointing a backward pass contains one more forward pass).

Forward keeps only the INPUT of every layer (the checkpoint); nothing else survives a layer.
Backward walks the layers from last to first: it recomputes the layer's forward pass from its
checkpoint, then computes the layer's gradients from the recomputed tensors; the gradient with
respect to the layer's input is the output gradient of the layer before it (the tensor the
paper keeps in its "conjunction buffer").  Recomputing changes no value: the result is the plain
chain rule through L layers, which is what the pins check.

Test infrastructure only.
"""
import numpy as np

from . import layer as _layer

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
GRAD_NAMES = tuple("d_" + k for k in PARAM_NAMES)


def forward(params, x, b, s, n, causal=True, counter=None):
    """params: list of L dicts with PARAM_NAMES; x [b*s, h].
    Returns (out, checkpoints) with checkpoints[l] = input of layer l."""
    cur = np.asarray(x, dtype=np.float64)
    checkpoints = []
    for p in params:
        checkpoints.append(cur)
        f = _layer.forward(dict(p, x=cur), b, s, n, causal=causal, keep_probs=False)
        if counter is not None:
            counter["forward_passes"] = counter.get("forward_passes", 0) + 1
        cur = f["out"]
    return cur, checkpoints


def backward(params, checkpoints, d_out, b, s, n, causal=True, counter=None):
    """Returns (d_x, grads) with grads[l] = dict of GRAD_NAMES for layer l."""
    g_out = np.asarray(d_out, dtype=np.float64)
    grads = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        inp = dict(params[l], x=checkpoints[l], d_out=g_out)
        f = _layer.forward(inp, b, s, n, causal=causal, keep_probs=False)   # the recomputation
        if counter is not None:
            counter["forward_passes"] = counter.get("forward_passes", 0) + 1
        g = _layer.backward(inp, f, b, s, n, causal=causal)
        grads[l] = {k: g[k] for k in GRAD_NAMES}
        g_out = g["d_x"]
    return g_out, grads
