"""GPU integration: every entry point in one chain -- tokens -> 2D embedding -> checkpointed stack of layers ->
final 2D LayerNorm -> lm-head (C = A B^T with the embedding table) -> 2D cross entropy, and the whole way back to the
table gradient -- against the same chain composed from the oracle's functions."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import layernorm as oln, model_ends as me, stack as ostack
from oracle.metrics import rel_frobenius
from workloads import LayerShape, layer_inputs, round_to_bf16, token_inputs
from gpu_util import mat_to_dev, mat_to_host, to_host, vec_to_dev, empty
from layer_util import TOL_BEHIND_LOGITS

pytestmark = pytest.mark.gpu
MATS = ("w_qkv", "w_o", "w1", "w2")
VEC_MULT = {"d_b_qkv": 3, "d_b_o": 1, "d_b1": 4, "d_b2": 1, "d_ln1_g": 1, "d_ln1_b": 1, "d_ln2_g": 1, "d_ln2_b": 1}


@pytest.mark.parametrize("fused", [False, True], ids=["probs", "fused"])
def test_tokens_to_loss_and_back(fused):
    shp, L, v = LayerShape(b=4, s=64, h=256, n=4, q=2), 2, 512
    M, h, q = shp.M, shp.h, shp.q
    rng = np.random.default_rng(17)
    tokens, labels = token_inputs(18, shp.b, shp.s, v)
    table = round_to_bf16((rng.standard_normal((v, h)) * 0.5).astype(np.float32))
    lnf_g = round_to_bf16((1.0 + 0.1 * rng.standard_normal(h)).astype(np.float32))
    lnf_b = round_to_bf16((0.1 * rng.standard_normal(h)).astype(np.float32))
    layers = []
    for l in range(L):
        inp = layer_inputs(40 + l, shp, "bf16", perturb_affine=True)
        for k in MATS:
            inp[k] = round_to_bf16(inp[k] * 4.0)
        layers.append({k: inp[k] for k in ostack.PARAM_NAMES})

    # ---- oracle chain (exact fp64 arithmetic on the same bf16 inputs) ----
    x0 = me.embedding(tokens, table)
    hid, ck = ostack.forward(layers, x0, shp.b, shp.s, shp.n, True)
    y, xhat, rstd = oln.forward(hid, lnf_g, lnf_b)
    logits = me.lm_head(y, table)
    loss_o, _ = me.cross_entropy(logits, labels)
    g_logits = me.cross_entropy_grad(logits, labels, 1.0 / M)
    g_y = g_logits @ table.astype(np.float64)
    g_table_head = g_logits.T @ y
    g_hid, g_lnf_g, g_lnf_b = oln.backward(g_y, xhat, rstd, lnf_g)
    g_x0, grads_o = ostack.backward(layers, ck, g_hid, shp.b, shp.s, shp.n, True)
    g_table = g_table_head + me.embedding_grad(tokens, g_x0, v)

    # ---- device chain ----
    cfg = opt.LayerCfg(shp.b, shp.s, shp.h, shp.n, shp.q, 1e-5, 1, opt.BF16, 1 if fused else 0)
    dTok = torch.from_numpy(tokens).to("cuda:0")
    dLab = torch.from_numpy(labels).to("cuda:0")
    dT = mat_to_dev(table, q, "bf16")
    P = []
    keep = []
    for p in layers:
        t = {k: mat_to_dev(p[k], q, "bf16") for k in MATS}
        t.update({k: vec_to_dev(p[k]) for k in ostack.PARAM_NAMES if k not in MATS})
        keep.append(t)
        P.append(opt.make_layer_params(t))
    sz = opt.stack_sizes(cfg, L)
    raw = {k: torch.empty(getattr(sz, k), dtype=torch.uint8, device="cuda:0")
           for k in ("workspace", "forward", "backward", "conjunction", "checkpoint")}
    buf = opt.make_stack_buffers(raw["workspace"], raw["forward"], raw["backward"], raw["conjunction"], raw["checkpoint"])
    rows = M // q
    X0, HID, Y, XH = (empty(M * h, "bf16") for _ in range(4))
    RSTD, ST, BST = empty(q * q * rows, "fp32"), empty(q * q * rows * 2, "fp32"), empty(q * q * rows * 2, "fp32")
    G, Bv = vec_to_dev(lnf_g), vec_to_dev(lnf_b)
    LOGITS, DLOG = empty(M * v, "bf16"), empty(M * v, "bf16")
    LOSS, LSE, CST = empty(q * q * rows, "fp32"), empty(q * q * rows, "fp32"), empty(q * q * rows * 2, "fp32")
    opt.embedding_fwd(dTok, dT, X0, M, v, h, q, -1, -1, opt.BF16)
    opt.stack_fwd(cfg, P, X0, buf, HID)
    opt.layernorm2d(HID, G, Bv, Y, XH, RSTD, ST, M, h, q, -1, -1, 1e-5, opt.BF16)
    opt.summa("abt", Y, dT, LOGITS, M, h, v, q, -1, -1, opt.BF16)
    opt.cross_entropy2d(LOGITS, dLab, LOSS, LSE, CST, M, v, q, -1, -1, opt.BF16)
    opt.cross_entropy2d_bwd(LOGITS, dLab, LSE, DLOG, 1.0 / M, M, v, q, -1, -1, opt.BF16)
    DY, DHID, DX0 = (empty(M * h, "bf16") for _ in range(3))
    DT_HEAD, DT_EMB = empty(v * h, "fp32"), empty(v * h, "fp32")
    DG, DB = empty(q * h, "fp32"), empty(q * h, "fp32")
    opt.summa("ab", DLOG, dT, DY, M, v, h, q, -1, -1, opt.BF16)
    opt.summa_ex("atb", DLOG, Y, DT_HEAD, v, M, h, q, -1, -1, opt.BF16, out_fp32=True)
    opt.layernorm2d_bwd(DY, XH, RSTD, G, None, DHID, DG, DB, BST, M, h, q, -1, -1, opt.BF16)
    grads = []
    for _ in range(L):
        g = {"d_w_qkv": empty(3 * h * h, "fp32"), "d_w_o": empty(h * h, "fp32"), "d_w1": empty(4 * h * h, "fp32"),
             "d_w2": empty(4 * h * h, "fp32")}
        g.update({k: empty(q * m * h, "fp32") for k, m in VEC_MULT.items()})
        grads.append(g)
    opt.stack_bwd(cfg, P, [opt.make_layer_grads(g) for g in grads], DHID, buf, DX0)
    opt.embedding_bwd(dTok, DX0, DT_EMB, M, v, h, q, -1, -1, opt.BF16)
    torch.cuda.synchronize()

    err = {}
    err["x0"] = rel_frobenius(mat_to_host(X0, M, h, q), x0)
    err["hidden"] = rel_frobenius(mat_to_host(HID, M, h, q), hid)
    err["logits"] = rel_frobenius(mat_to_host(LOGITS, M, v, q), logits)
    got_loss = to_host(LOSS).reshape(q, q, rows)[:, 0].reshape(-1)
    err["mean_loss"] = abs(got_loss.mean() - loss_o.mean()) / abs(loss_o.mean())
    err["d_hidden"] = rel_frobenius(mat_to_host(DHID, M, h, q), g_hid)
    err["d_x0"] = rel_frobenius(mat_to_host(DX0, M, h, q), g_x0)
    err["d_lnf_g"] = rel_frobenius(to_host(DG).reshape(q, q, -1).sum(axis=0).reshape(-1), g_lnf_g)
    err["d_table"] = rel_frobenius(mat_to_host(DT_HEAD, v, h, q).astype(np.float64) + mat_to_host(DT_EMB, v, h, q), g_table)
    for l in range(L):
        err[f"L{l}.d_w1"] = rel_frobenius(mat_to_host(grads[l]["d_w1"], h, 4 * h, q), grads_o[l]["d_w1"])
        err[f"L{l}.d_w_qkv"] = rel_frobenius(mat_to_host(grads[l]["d_w_qkv"], h, 3 * h, q), grads_o[l]["d_w_qkv"])
    print("tokens -> loss -> table gradient, relative errors against the exact oracle chain:", {k: f"{e:.1e}" for k, e in err.items()})
    assert err["x0"] == 0.0
    # Exact-oracle chain bound: as for the stack (tests of the stack), with the two model ends counted as one more
    # layer: TOL_BEHIND_LOGITS * sqrt(2 (L + 1)).
    tol = TOL_BEHIND_LOGITS * float(np.sqrt(2 * (L + 1)))
    assert all(e <= tol for e in err.values()), err
    assert err["mean_loss"] <= 5e-3
