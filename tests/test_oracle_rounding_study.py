"""The bf16-storage error budget (oracle/rounding_study.py): pinned to the oracle, and the facts the GPU tests'
per-tensor bounds rest on."""
import numpy as np

from oracle import layer, rounding_study as rs
from oracle.metrics import rel_frobenius
from workloads import LayerShape, layer_inputs, round_to_bf16


def _inputs(seed=3):
    """A small layer whose soft-max logits have the scale of the 4096-wide benchmark layers (standard deviation
    about 1.6: activations N(0,1), weights N(0, 0.02^2), h = 4096 -> q, k entries of std 1.28): h = 256 with the
    weights scaled by sqrt(4096 / 256)."""
    shp = LayerShape(b=2, s=128, h=256, n=4, q=1)
    inp = layer_inputs(seed, shp, "bf16", perturb_affine=False)
    for k in ("w_qkv", "w_o", "w1", "w2"):
        inp[k] = round_to_bf16(inp[k] * 4.0)
    return shp, inp


def test_nothing_rounded_is_the_oracle():
    shp, inp = _inputs()
    f = layer.forward(inp, shp.b, shp.s, shp.n)
    g = layer.backward(inp, f, shp.b, shp.s, shp.n)
    t = rs.layer(inp, shp.b, shp.s, shp.n, rounded=())
    for k in ("ln1_out", "qkv", "attn", "h_mid", "pre_gelu", "gelu", "out"):
        assert np.allclose(t[k], f[k], rtol=0, atol=1e-12), k
    for k in ("d_pre_gelu", "d_h_mid", "d_attn", "d_qkv", "d_ln1_out", "d_x", "d_w_qkv", "d_w_o", "d_w1", "d_w2", "d_ln1_g"):
        assert np.allclose(t[k], g[k], rtol=0, atol=1e-10), k


def test_a_rounded_tensor_is_bf16_and_later_stages_read_it():
    shp, inp = _inputs()
    t = rs.layer(inp, shp.b, shp.s, shp.n, rounded=("qkv",))
    v = t["qkv"].astype(np.float32)
    assert np.array_equal(round_to_bf16(v), v)
    exact = rs.layer(inp, shp.b, shp.s, shp.n)
    assert np.array_equal(t["ln1_out"], exact["ln1_out"])          # upstream untouched
    assert 0 < rel_frobenius(t["attn"], exact["attn"]) < 1e-2      # downstream moved


def test_logit_operands_alone_exceed_5e3_behind_the_softmax():
    """Rounding ONLY the two operands that feed the logits (LayerNorm-1 output into the QKV product, Q/K into
    QK^T) already moves the gradients behind the attention by more than 5e-3 at the benchmark layers' logit
    scale; with every stored tensor rounded they land at 6.3-7.6e-3, below the bound the GPU tests use for them
    (9e-3), while everything else stays near or below 5e-3 (on the benchmark layers themselves the GPU tests
    measure it: <= 4.9e-3)."""
    shp, inp = _inputs()
    exact = rs.layer(inp, shp.b, shp.s, shp.n)
    two = rs.layer(inp, shp.b, shp.s, shp.n, rounded=("ln1_out", "qkv"))
    for k in ("d_qkv", "d_ln1_out", "d_w_qkv"):
        e = rel_frobenius(two[k], exact[k])
        assert 5e-3 < e < 6.5e-3, (k, e)
    every = rs.layer(inp, shp.b, shp.s, shp.n, rounded=rs.TENSORS)
    errs = {k: rel_frobenius(every[k], exact[k]) for k in exact if k not in ("rstd1", "rstd2")}
    behind = ("d_qkv", "d_ln1_out", "d_x", "d_w_qkv", "d_w_o", "d_ln1_g", "d_ln1_b")
    for k, e in errs.items():
        assert e < (9e-3 if k in behind else 5.2e-3), (k, e, errs)
    assert max(errs[k] for k in behind) > 6.5e-3
    # before the attention nothing is amplified: one or two roundings deep
    for k in ("ln1_out", "xhat1", "qkv"):
        assert errs[k] < 2.5e-3, (k, errs[k])


def test_a_wider_qkv_alone_would_not_reach_5e3():
    """qkv is not an operand of a SUMMA product, so it could be stored wider than bf16; with qkv exact and every other
    stored tensor rounded the gradients behind the logits still exceed 5e-3 (the LayerNorm-1 output, which IS a bf16
    SUMMA operand, contributes as much as qkv does)."""
    shp, inp = _inputs()
    exact = rs.layer(inp, shp.b, shp.s, shp.n)
    t = rs.layer(inp, shp.b, shp.s, shp.n, rounded=tuple(k for k in rs.TENSORS if k != "qkv"))
    for k in ("d_qkv", "d_ln1_out", "d_w_qkv"):
        assert rel_frobenius(t[k], exact[k]) > 5.5e-3, k
    one_a = rs.layer(inp, shp.b, shp.s, shp.n, rounded=("ln1_out",))
    one_b = rs.layer(inp, shp.b, shp.s, shp.n, rounded=("qkv",))
    ea, eb = rel_frobenius(one_a["d_qkv"], exact["d_qkv"]), rel_frobenius(one_b["d_qkv"], exact["d_qkv"])
    assert 0.8 < ea / eb < 1.25, (ea, eb)
