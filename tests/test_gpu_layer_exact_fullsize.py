"""GPU parity of the WHOLE layer at the full sizes of benchmark configurations 4 and 5 against the unpartitioned
fp64 oracle (Fig. 4's layer, Eq. 1, Section 3.2): every forward tensor, every activation gradient and every
parameter gradient, whole tensors, every block.

Configuration 4 (b=8, s=1024, h=4096, 32 heads, q=4): the oracle computes the whole logical layer (about 10 TFLOP
of host work, under a minute on the machine's cores).  The same run shows that restricting the oracle to the sequences
of one block row changes nothing for that block row's forward tensors and activation gradients (every operation
of the layer acts on rows or on whole sequences independently); configuration 5 (b=64, s=512, h=4096, q=8; the
whole logical layer would be 40 TFLOP of host work) is then checked on one block row that way.
"""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import layer as olayer
from oracle.metrics import rel_frobenius
from workloads import CONFIGS, LayerShape, layer_inputs
from gpu_util import to_host
from layer_util import alloc_layer, bound, compare_all, fetch, FWD_OUT, BWD_OUT

pytestmark = pytest.mark.gpu
ROW_LOCAL = FWD_OUT + BWD_OUT      # tensors whose rows depend on the rows of the same sequences only


def _rows_only(inp, rows):
    """The layer inputs restricted to a range of rows (whole sequences): parameters unchanged."""
    sub = dict(inp)
    sub["x"], sub["d_out"] = inp["x"][rows], inp["d_out"][rows]
    return sub


def test_config4_whole_layer_against_the_exact_oracle():
    shp = CONFIGS["config4"]["layer"]
    inp = layer_inputs(CONFIGS["config4"]["seed"], shp, "bf16", perturb_affine=True)
    cfg, T, lt, ws = alloc_layer(inp, shp, True)
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    print("config4: device pass done, oracle running", flush=True)
    fe = olayer.forward(inp, shp.b, shp.s, shp.n, causal=True, keep_probs=False)
    be = olayer.backward(inp, fe, shp.b, shp.s, shp.n, causal=True)
    errs = compare_all(T, shp, inp, fe, be, check=False)
    print("config4 whole layer vs exact oracle:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: (v, bound(k)) for k, v in errs.items() if not v <= bound(k)}
    assert not bad, bad

    # the oracle restricted to block row i's sequences equals the full oracle on those rows
    i, q = 2, shp.q
    rows = slice(i * shp.M // q, (i + 1) * shp.M // q)
    sub = _rows_only(inp, rows)
    fr = olayer.forward(sub, shp.b // q, shp.s, shp.n, causal=True, keep_probs=False)
    br = olayer.backward(sub, fr, shp.b // q, shp.s, shp.n, causal=True)
    for k in FWD_OUT:
        assert rel_frobenius(fr[k], fe[k][rows]) <= 1e-12, k
    for k in BWD_OUT:
        assert rel_frobenius(br[k], be[k][rows]) <= 1e-12, k


def test_config5_block_row_against_the_exact_oracle():
    shp = CONFIGS["config5"]["layer"]
    q, i = shp.q, 5
    inp = layer_inputs(CONFIGS["config5"]["seed"], shp, "bf16", perturb_affine=True)
    cfg, T, lt, ws = alloc_layer(inp, shp, True)
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()
    print("config5: device pass done, oracle running on block row", i, flush=True)
    rows = slice(i * shp.M // q, (i + 1) * shp.M // q)
    sub = _rows_only(inp, rows)
    fr = olayer.forward(sub, shp.b // q, shp.s, shp.n, causal=True, keep_probs=False)
    br = olayer.backward(sub, fr, shp.b // q, shp.s, shp.n, causal=True)
    errs = {}
    for k in FWD_OUT:
        errs[k] = rel_frobenius(fetch(T, k, shp)[rows], fr[k])
    for k in BWD_OUT:
        errs[k] = rel_frobenius(fetch(T, k, shp)[rows], br[k])
    rb = shp.M // q
    for k in ("1", "2"):
        errs["rstd" + k] = rel_frobenius(to_host(T["rstd" + k]).reshape(q, q, rb)[i], np.tile(fr["rstd" + k], (q, 1)))
    print(f"config5 block row {i} vs exact oracle:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: (v, bound(k)) for k, v in errs.items() if not v <= bound(k)}
    assert not bad, bad
