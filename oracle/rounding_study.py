"""Error budget of bf16 storage along the layer: NOT an oracle and never compared with device results.

The layer of oracle.layer (Sections 2.1 and 3.2, Eq. 1) is evaluated in fp64 once more, with the one difference
that the tensors named by the caller are rounded to bf16 (nearest even) at the moment they are produced, so that
every later stage reads the rounded value.  Comparing its result with oracle.layer's says how much of the
distance between ANY implementation that keeps those tensors in bf16 and real arithmetic is due to the storage
format alone, and which tensor contributes what.  The tests use it for one purpose: to show that the bound they
hold the gradients behind the soft-max logits to cannot be 5e-3 once the operands of the matrix products are
bf16 (tests/test_oracle_rounding_study.py), i.e. to justify a tolerance -- no device tensor is ever compared
with anything computed here.

Test infrastructure only.
"""
import numpy as np

from workloads import round_to_bf16

from . import attention as _att
from . import layer as _layer
from . import layernorm as _ln

# every tensor of the layer that could be kept in a 16-bit format ("d_scores" = dS inside the attention backward)
TENSORS = ("ln1_out", "xhat1", "qkv", "probs", "attn", "h_mid", "ln2_out", "xhat2", "pre_gelu", "gelu", "out",
           "d_pre_gelu", "d_ln2_out", "d_h_mid", "d_attn", "d_scores", "d_qkv", "d_ln1_out", "d_x")


def _f(t):
    return np.asarray(t, dtype=np.float64)


def layer(inp, b, s, n, rounded=(), causal=True, eps=_ln.EPS_DEFAULT):
    """Forward and backward of one layer with the tensors in ``rounded`` passed through bf16 when produced.
    Returns one dict with the forward tensors and the gradients (names of oracle.layer)."""
    unknown = set(rounded) - set(TENSORS)
    if unknown:
        raise ValueError(f"unknown tensors {sorted(unknown)}")

    def r(name, v):
        return round_to_bf16(np.asarray(v, dtype=np.float32)).astype(np.float64) if name in rounded else v

    x = _f(inp["x"])
    h = x.shape[1]
    d = h // n
    t = {}
    y, xhat, t["rstd1"] = _ln.forward(x, inp["ln1_g"], inp["ln1_b"], eps)
    t["ln1_out"], t["xhat1"] = r("ln1_out", y), r("xhat1", xhat)
    t["qkv"] = r("qkv", t["ln1_out"] @ _f(inp["w_qkv"]) + _f(inp["b_qkv"])[None, :])
    attn = np.empty((b * s, h))
    probs = {}
    for seq in range(b):
        for head in range(n):
            Q, K, V = _att.split_qkv(t["qkv"], b, s, n, seq, head)
            _, P = _att.head_forward(Q, K, V, causal)
            P = r("probs", P)
            probs[seq, head] = P
            attn[seq * s:(seq + 1) * s, head * d:(head + 1) * d] = P @ V
    t["attn"] = r("attn", attn)
    t["h_mid"] = r("h_mid", x + t["attn"] @ _f(inp["w_o"]) + _f(inp["b_o"])[None, :])
    y, xhat, t["rstd2"] = _ln.forward(t["h_mid"], inp["ln2_g"], inp["ln2_b"], eps)
    t["ln2_out"], t["xhat2"] = r("ln2_out", y), r("xhat2", xhat)
    pre = t["ln2_out"] @ _f(inp["w1"]) + _f(inp["b1"])[None, :]
    t["pre_gelu"] = r("pre_gelu", pre)
    t["gelu"] = r("gelu", _layer.gelu(pre))
    t["out"] = r("out", t["h_mid"] + t["gelu"] @ _f(inp["w2"]) + _f(inp["b2"])[None, :])

    d_out = _f(inp["d_out"])
    t["d_w2"] = t["gelu"].T @ d_out
    t["d_pre_gelu"] = r("d_pre_gelu", (d_out @ _f(inp["w2"]).T) * _layer.gelu_grad(t["pre_gelu"]))
    t["d_ln2_out"] = r("d_ln2_out", t["d_pre_gelu"] @ _f(inp["w1"]).T)
    t["d_w1"] = t["ln2_out"].T @ t["d_pre_gelu"]
    dx2, t["d_ln2_g"], t["d_ln2_b"] = _ln.backward(t["d_ln2_out"], t["xhat2"], t["rstd2"], inp["ln2_g"])
    t["d_h_mid"] = r("d_h_mid", d_out + dx2)
    t["d_attn"] = r("d_attn", t["d_h_mid"] @ _f(inp["w_o"]).T)
    t["d_w_o"] = t["attn"].T @ t["d_h_mid"]
    d_qkv = np.empty_like(t["qkv"])
    for seq in range(b):
        for head in range(n):
            Q, K, V = _att.split_qkv(t["qkv"], b, s, n, seq, head)
            P = probs[seq, head]
            dO = t["d_attn"][seq * s:(seq + 1) * s, head * d:(head + 1) * d]
            dP = dO @ V.T
            dS = r("d_scores", P * (dP - (dP * P).sum(axis=1, keepdims=True)))
            rows, c0 = slice(seq * s, (seq + 1) * s), head * 3 * d
            d_qkv[rows, c0:c0 + d] = dS @ K / np.sqrt(d)
            d_qkv[rows, c0 + d:c0 + 2 * d] = dS.T @ Q / np.sqrt(d)
            d_qkv[rows, c0 + 2 * d:c0 + 3 * d] = P.T @ dO
    t["d_qkv"] = r("d_qkv", d_qkv)
    t["d_ln1_out"] = r("d_ln1_out", t["d_qkv"] @ _f(inp["w_qkv"]).T)
    t["d_w_qkv"] = t["ln1_out"].T @ t["d_qkv"]
    dx1, t["d_ln1_g"], t["d_ln1_b"] = _ln.backward(t["d_ln1_out"], t["xhat1"], t["rstd1"], inp["ln1_g"])
    t["d_x"] = r("d_x", t["d_h_mid"] + dx1)
    return t
