"""One transformer layer, unpartitioned, fp64 (Sections 2.1, 3.2; Eq. 1).

Wiring (the paper's figures omit residuals, normalisation and non-linearities;
this is the pre-LayerNorm layer of the system it is compared with):

  a1   = LN1(x)                       h_mid = x + attn @ w_o + b_o
  qkv  = a1 @ w_qkv + b_qkv           a2    = LN2(h_mid)
  attn = softmax(QK^T/sqrt(d)) V      z     = a2 @ w1 + b1 ; g = GeLU(z)
                                      out   = h_mid + g @ w2 + b2

GeLU is the exact form x * Phi(x).  No dropout.  Backward uses the saved
forward tensors (no recomputation): every linear follows Eq. 1
(dX = dY W^T, dW = X^T dY, db = column sums of dY).

Every intermediate stays in fp64: nothing is rounded anywhere.

Test infrastructure only.
"""
import math

import numpy as np
from scipy.special import erf as _erf  # library primitive; pinned against math.erf in the tests

from . import attention as _att
from . import layernorm as _ln


def gelu(z):
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_grad(z):
    z = np.asarray(z, dtype=np.float64)
    cdf = 0.5 * (1.0 + _erf(z / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    return cdf + z * pdf


def _f(t):
    return np.asarray(t, dtype=np.float64)


def forward(inp, b, s, n, causal=True, eps=_ln.EPS_DEFAULT, keep_probs=True):
    """inp: dict of logical tensors (see workloads.layer_inputs). Returns dict of every stage."""
    x = _f(inp["x"])
    t = {}
    t["ln1_out"], t["xhat1"], t["rstd1"] = _ln.forward(x, inp["ln1_g"], inp["ln1_b"], eps)
    t["qkv"] = t["ln1_out"] @ _f(inp["w_qkv"]) + _f(inp["b_qkv"])[None, :]
    t["attn"], t["probs"] = _att.forward(t["qkv"], b, s, n, causal, keep_probs)
    t["h_mid"] = x + t["attn"] @ _f(inp["w_o"]) + _f(inp["b_o"])[None, :]
    t["ln2_out"], t["xhat2"], t["rstd2"] = _ln.forward(t["h_mid"], inp["ln2_g"], inp["ln2_b"], eps)
    t["pre_gelu"] = t["ln2_out"] @ _f(inp["w1"]) + _f(inp["b1"])[None, :]
    t["gelu"] = gelu(t["pre_gelu"])
    t["out"] = t["h_mid"] + t["gelu"] @ _f(inp["w2"]) + _f(inp["b2"])[None, :]
    return t


def backward(inp, fwd, b, s, n, causal=True):
    """Gradients of <d_out, out> w.r.t. x and every parameter, plus intermediate gradients."""
    d_out = _f(inp["d_out"])
    g = {}
    # out = h_mid + gelu @ w2 + b2
    g["d_gelu"] = d_out @ _f(inp["w2"]).T
    g["d_w2"] = fwd["gelu"].T @ d_out
    g["d_b2"] = d_out.sum(axis=0)
    g["d_pre_gelu"] = g["d_gelu"] * gelu_grad(fwd["pre_gelu"])
    # pre_gelu = ln2_out @ w1 + b1
    g["d_ln2_out"] = g["d_pre_gelu"] @ _f(inp["w1"]).T
    g["d_w1"] = fwd["ln2_out"].T @ g["d_pre_gelu"]
    g["d_b1"] = g["d_pre_gelu"].sum(axis=0)
    dx2, g["d_ln2_g"], g["d_ln2_b"] = _ln.backward(g["d_ln2_out"], fwd["xhat2"], fwd["rstd2"], inp["ln2_g"])
    g["d_h_mid"] = d_out + dx2
    # h_mid = x + attn @ w_o + b_o
    g["d_attn"] = g["d_h_mid"] @ _f(inp["w_o"]).T
    g["d_w_o"] = fwd["attn"].T @ g["d_h_mid"]
    g["d_b_o"] = g["d_h_mid"].sum(axis=0)
    g["d_qkv"] = _att.backward(fwd["qkv"], g["d_attn"], b, s, n, causal)
    # qkv = ln1_out @ w_qkv + b_qkv
    g["d_ln1_out"] = g["d_qkv"] @ _f(inp["w_qkv"]).T
    g["d_w_qkv"] = fwd["ln1_out"].T @ g["d_qkv"]
    g["d_b_qkv"] = g["d_qkv"].sum(axis=0)
    dx1, g["d_ln1_g"], g["d_ln1_b"] = _ln.backward(g["d_ln1_out"], fwd["xhat1"], fwd["rstd1"], inp["ln1_g"])
    g["d_x"] = g["d_h_mid"] + dx1
    return g
