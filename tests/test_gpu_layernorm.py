"""GPU parity: 2D LayerNorm forward/backward through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import blocks, layernorm as oln
from oracle.metrics import rel_frobenius
from workloads import round_to_bf16
from gpu_util import to_dev, to_host, mat_to_dev, mat_to_host, vec_to_dev, empty, dt

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-5, "bf16": 5e-3}
EPS = 1e-5


def _inputs(seed, M, H, dtype):
    rng = np.random.default_rng(seed)
    rnd = round_to_bf16 if dtype == "bf16" else (lambda v: v.astype(np.float32))
    x = rnd((rng.standard_normal((M, H)) * 1.5 + 0.3).astype(np.float32))
    gamma = rnd((1.0 + 0.2 * rng.standard_normal(H)).astype(np.float32))
    beta = rnd((0.1 * rng.standard_normal(H)).astype(np.float32))
    dy = rnd(rng.standard_normal((M, H)).astype(np.float32))
    dres = rnd(rng.standard_normal((M, H)).astype(np.float32))
    return x, gamma, beta, dy, dres


# (M, H, q): vector path, ragged columns (scalar path), wide rows (re-read path), q = 1; workgroups of 1, 2 and 4
# rows per grid row (odd row counts), q = 3 and 8 wavefronts per row, and q = 32 (more wavefronts than a workgroup
# holds: statistics kernel first, then the apply kernel)
CASES = [(64, 512, 2), (36, 100, 2), (24, 8192 * 2, 2), (16, 96, 1), (48, 768, 4), (10, 4096, 1),
         (18, 128, 2), (96, 384, 3), (40, 512, 8), (64, 1024, 32)]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("M,H,q", CASES)
def test_forward_backward_grid(M, H, q, dtype):
    x, gamma, beta, dy, dres = _inputs(M + H, M, H, dtype)
    y_o, xhat_o, rstd_o = oln.forward(x, gamma, beta, EPS)
    rows, cols = M // q, H // q
    dX = mat_to_dev(x, q, dtype)
    dG, dB = vec_to_dev(gamma), vec_to_dev(beta)
    Y, XH = empty(M * H, dtype), empty(M * H, dtype)
    rstd, stats = empty(q * q * rows, "fp32"), empty(q * q * rows * 2, "fp32")
    opt.layernorm2d(dX, dG, dB, Y, XH, rstd, stats, M, H, q, -1, -1, EPS, dt(dtype))
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_frobenius(mat_to_host(Y, M, H, q), y_o) <= tol
    assert rel_frobenius(mat_to_host(XH, M, H, q), xhat_o) <= tol
    r = to_host(rstd).reshape(q, q, rows)
    st = to_host(stats).reshape(q, q, rows, 2)
    for i in range(q):
        for j in range(q):
            assert rel_frobenius(r[i, j], rstd_o[i * rows:(i + 1) * rows]) <= 1e-5
            assert rel_frobenius(st[i, j], oln.partial_stats(x, q, i, j)) <= 1e-5
    # zero mean / unit variance of the normalised rows (the oracle's invariant, checked on the GPU output)
    xh = mat_to_host(XH, M, H, q).astype(np.float64)
    assert np.all(np.abs(xh.mean(axis=1)) < (2e-2 if dtype == "bf16" else 1e-4))
    assert np.all(np.abs(xh.var(axis=1) - 1.0) < (2e-2 if dtype == "bf16" else 1e-3))

    # backward, with the saved xhat/rstd the GPU produced replaced by the oracle's (rounded to storage) so the
    # comparison isolates the backward arithmetic
    xh_in = (round_to_bf16(xhat_o.astype(np.float32)) if dtype == "bf16" else xhat_o.astype(np.float32))
    rstd_in = np.tile(rstd_o.astype(np.float32).reshape(q, 1, rows), (1, q, 1))
    dx_o, dg_o, db_o = oln.backward(dy, xh_in, rstd_in[:, 0].reshape(-1), gamma)
    dXH, dDY, dRES = mat_to_dev(xh_in, q, dtype), mat_to_dev(dy, q, dtype), mat_to_dev(dres, q, dtype)
    DX = empty(M * H, dtype)
    dgp, dbp = empty(q * q * cols, "fp32"), empty(q * q * cols, "fp32")
    bst = empty(q * q * rows * 2, "fp32")
    opt.layernorm2d_bwd(dDY, dXH, to_dev(rstd_in, "fp32"), dG, dRES, DX, dgp, dbp, bst, M, H, q, -1, -1, dt(dtype))
    torch.cuda.synchronize()
    assert rel_frobenius(mat_to_host(DX, M, H, q), dx_o + dres) <= tol
    g_part, b_part = to_host(dgp).reshape(q, q, cols), to_host(dbp).reshape(q, q, cols)
    # summing the partials over the grid rows is the reduce to row 0
    ptol = 1e-5 if dtype == "fp32" else 1e-4      # fp32 path: 1e-5; bf16 inputs summed in fp32
    assert rel_frobenius(g_part.sum(axis=0).reshape(-1), dg_o) <= ptol
    assert rel_frobenius(b_part.sum(axis=0).reshape(-1), db_o) <= ptol
    for i in range(q):
        for j in range(q):
            rs, cs = slice(i * rows, (i + 1) * rows), slice(j * cols, (j + 1) * cols)
            want = (dy[rs, cs].astype(np.float64) * xh_in[rs, cs]).sum(axis=0)
            assert rel_frobenius(g_part[i, j], want) <= ptol
    # without the residual-branch gradient
    DX2 = empty(M * H, dtype)
    opt.layernorm2d_bwd(dDY, dXH, to_dev(rstd_in, "fp32"), dG, None, DX2, None, None, bst, M, H, q, -1, -1, dt(dtype))
    torch.cuda.synchronize()
    assert rel_frobenius(mat_to_host(DX2, M, H, q), dx_o) <= tol


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_device_mode_uses_resident_peer_stats(dtype):
    """Device (i, j) computes its own partial and adds the peers' resident partials: same bits as grid mode."""
    M, H, q = 32, 1024, 4
    rows, cols = M // q, H // q
    x, gamma, beta, dy, dres = _inputs(5, M, H, dtype)
    dX, dG, dB = mat_to_dev(x, q, dtype), vec_to_dev(gamma), vec_to_dev(beta)
    Yg, XHg = empty(M * H, dtype), empty(M * H, dtype)
    rstd_g, stats = empty(q * q * rows, "fp32"), empty(q * q * rows * 2, "fp32")
    opt.layernorm2d(dX, dG, dB, Yg, XHg, rstd_g, stats, M, H, q, -1, -1, EPS, dt(dtype))
    i, j = 2, 1
    # peers' partials via the explicit per-device stats call into a fresh buffer
    stats2 = empty(q * q * rows * 2, "fp32")
    for l in range(q):
        if l != j:
            opt.layernorm2d_stats(dX, stats2, M, H, q, i, l, dt(dtype))
    Yd, XHd, rstd_d = empty(M * H, dtype), empty(M * H, dtype), empty(q * q * rows, "fp32")
    opt.layernorm2d(dX, dG, dB, Yd, XHd, rstd_d, stats2, M, H, q, i, j, EPS, dt(dtype))
    torch.cuda.synchronize()
    blk = slice((i * q + j) * rows * cols, (i * q + j + 1) * rows * cols)
    assert np.array_equal(to_host(Yd)[blk], to_host(Yg)[blk])
    assert np.array_equal(to_host(XHd)[blk], to_host(XHg)[blk])
    others = np.ones(M * H, dtype=bool)
    others[blk] = False
    assert np.all(np.isnan(to_host(Yd)[others]))
    s_g, s_d = to_host(stats).reshape(q, q, rows, 2), to_host(stats2).reshape(q, q, rows, 2)
    assert np.array_equal(s_g[i], s_d[i])                 # all q partials of grid row i now present
    assert np.all(np.isnan(s_d[(i + 1) % q]))             # other grid rows untouched
    # backward, device mode == grid mode
    dDY = mat_to_dev(dy, q, dtype)
    DXg, DXd = empty(M * H, dtype), empty(M * H, dtype)
    bst = empty(q * q * rows * 2, "fp32")
    opt.layernorm2d_bwd(dDY, XHg, rstd_g, dG, None, DXg, None, None, bst, M, H, q, -1, -1, dt(dtype))
    bst2 = empty(q * q * rows * 2, "fp32")
    for l in range(q):
        if l != j:
            opt.layernorm2d_bwd_stats(dDY, XHg, dG, bst2, M, H, q, i, l, dt(dtype))
    opt.layernorm2d_bwd(dDY, XHg, rstd_g, dG, None, DXd, None, None, bst2, M, H, q, i, j, dt(dtype))
    torch.cuda.synchronize()
    assert np.array_equal(to_host(DXd)[blk], to_host(DXg)[blk])


def test_constant_row_and_shift_invariance():
    """A constant row has zero variance: E[x^2]-E[x]^2 may round below 0 and must be clamped, output = beta."""
    M, H, q = 8, 256, 2
    x = np.full((M, H), 3.0, dtype=np.float32)
    x[1] = np.linspace(-1, 1, H, dtype=np.float32)
    gamma, beta = np.ones(H, np.float32), np.full(H, 0.5, np.float32)
    Y, XH = empty(M * H, "fp32"), empty(M * H, "fp32")
    rstd, stats = empty(q * q * (M // q), "fp32"), empty(q * q * (M // q) * 2, "fp32")
    opt.layernorm2d(mat_to_dev(x, q, "fp32"), vec_to_dev(gamma), vec_to_dev(beta), Y, XH, rstd, stats, M, H, q, -1, -1, EPS, opt.FP32)
    torch.cuda.synchronize()
    y = mat_to_host(Y, M, H, q)
    assert np.all(np.isfinite(y))
    assert np.allclose(y[0], 0.5, atol=1e-3)
    y_o, _, _ = oln.forward(x, gamma, beta, EPS)
    assert rel_frobenius(y[1], y_o[1]) <= 1e-5
