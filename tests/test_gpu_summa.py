"""GPU parity: the three SUMMA products through the C ABI against the fp64 oracle.

Tolerances (relative Frobenius error per block): 1e-5 on the fp32 path, 5e-3 for bf16 inputs with fp32
accumulation.  Integer-valued operands must come out bit-exact in any summation order.
"""
import numpy as np
import pytest
import torch

import paper_2104_05343_amd as opt
from oracle import blocks, summa, layer as olayer
from oracle.metrics import rel_frobenius
from workloads import gemm_inputs, gemm_cases, round_to_bf16
from gpu_util import to_dev, to_host, mat_to_dev, mat_to_host, vec_to_dev, empty, dt

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-5, "bf16": 5e-3}
FORMS = ["ab", "abt", "atb"]


def _run(form, A, B, M, K, N, q, dtype, i=-1, j=-1, ws=None, out=None):
    dA, dB = mat_to_dev(A, q, dtype), mat_to_dev(B, q, dtype)
    dC = empty(M * N, dtype) if out is None else out
    opt.summa(form, dA, dB, dC, M, K, N, q, i, j, dt(dtype), ws=ws)
    torch.cuda.synchronize()
    return dC


def _check_blocks(dC, want, M, N, q, tol, coords=None):
    got = to_host(dC).reshape(q, q, M // q, N // q)
    for i in range(q):
        for j in range(q):
            if coords is not None and (i, j) not in coords:
                assert np.all(np.isnan(got[i, j])), f"block ({i},{j}) was written but not requested"
                continue
            err = rel_frobenius(got[i, j], blocks.block(want, q, i, j))
            assert err <= tol, f"block ({i},{j}): rel Frobenius {err:.3e} > {tol}"


def test_config1_fp32_all_blocks():
    for g in gemm_cases("config1"):
        A, B = gemm_inputs(g.seed, g.form, g.M, g.K, g.N, g.dtype, g.dist_a, g.dist_b)
        want = summa.product(g.form, A, B)
        dC = _run(g.form, A, B, g.M, g.K, g.N, g.q, "fp32")
        _check_blocks(dC, want, g.M, g.N, g.q, TOL["fp32"])
        for (i, j) in [(0, 0), (0, 1), (1, 0), (1, 1)]:
            dC1 = _run(g.form, A, B, g.M, g.K, g.N, g.q, "fp32", i, j)
            _check_blocks(dC1, want, g.M, g.N, g.q, TOL["fp32"], coords={(i, j)})


def _int_operands(form, M, K, N):
    m, k, n = np.arange(M), np.arange(K), np.arange(N)
    A = ((m[:, None] * 3 + k[None, :] * 5) % 17 - 8).astype(np.float32)   # logical [M, K], |v| <= 8
    B = ((k[:, None] * 7 + n[None, :] * 2) % 13 - 6).astype(np.float32)   # logical [K, N]
    want = (A.astype(np.int64) @ B.astype(np.int64))
    if form == "abt":
        B = np.ascontiguousarray(B.T)
    if form == "atb":
        A = np.ascontiguousarray(A.T)
    return A, B, want


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("q", [1, 2, 4])
@pytest.mark.parametrize("form", FORMS)
def test_exact_integer_pattern(form, q, dtype):
    """Block indexing is bit-exact: small integers multiply and add exactly in fp32 (|sum| < 2^24)."""
    for (M, K, N) in [(8 * q, 16 * q, 12 * q), (136 * q, 72 * q, 200 * q), (256 * q, 64 * q, 128 * q)]:
        A, B, want = _int_operands(form, M, K, N)
        dC = _run(form, A, B, M, K, N, q, dtype)
        got = mat_to_host(dC, M, N, q)
        assert np.array_equal(got.astype(np.int64), want), (form, q, dtype, M, K, N)
        assert np.array_equal(got, want.astype(np.float32))
        i, j = q - 1, 0
        dC1 = _run(form, A, B, M, K, N, q, dtype, i, j)
        g1 = to_host(dC1).reshape(q, q, M // q, N // q)[i, j]
        assert np.array_equal(g1, blocks.block(want, q, i, j).astype(np.float32))


# per-block shapes: matrix-core fast path (multiples of the tile), bounds-checked matrix-core path
# (multiples of 8, ragged against the 128-tile), scalar path (odd sizes)
SHAPES = [(384, 192, 256), (200, 72, 136), (37, 19, 50), (512, 64, 128), (264, 520, 1032)]


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("q", [1, 2, 3])
def test_bf16_random_blocks(form, q):
    for si, (mb, kp, nb) in enumerate(SHAPES):
        M, K, N = mb * q, kp * q, nb * q
        A, B = gemm_inputs(100 + si, form, M, K, N, "bf16", "n1", "n1")
        want = summa.product(form, A, B)
        dC = _run(form, A, B, M, K, N, q, "bf16")
        _check_blocks(dC, want, M, N, q, TOL["bf16"])
        i, j = (q - 1, q // 2)
        dC1 = _run(form, A, B, M, K, N, q, "bf16", i, j)
        _check_blocks(dC1, want, M, N, q, TOL["bf16"], coords={(i, j)})
        # device mode and grid mode agree bit for bit on the block they share
        b_grid = to_host(dC).reshape(q, q, mb, nb)[i, j]
        b_dev = to_host(dC1).reshape(q, q, mb, nb)[i, j]
        assert np.array_equal(b_grid, b_dev)


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("kp", [32, 96, 64, 192, 320])
def test_bf16_short_and_odd_panel_lengths(form, kp):
    """Tile-multiple blocks whose panel length is an odd or even number of 32-slabs: odd counts cannot use the
    pair-wise k-loop and take the bounds-checked kernel; 64 is the shortest fast case (one pair per panel)."""
    q, mb, nb = 2, 256, 256
    M, K, N = mb * q, kp * q, nb * q
    A, B = gemm_inputs(300 + kp, form, M, K, N, "bf16", "n1", "n1")
    want = summa.product(form, A, B)
    dC = _run(form, A, B, M, K, N, q, "bf16")
    _check_blocks(dC, want, M, N, q, TOL["bf16"])
    dC1 = _run(form, A, B, M, K, N, q, "bf16", 1, 0)
    _check_blocks(dC1, want, M, N, q, TOL["bf16"], coords={(1, 0)})
    assert np.array_equal(to_host(dC).reshape(q, q, mb, nb)[1, 0], to_host(dC1).reshape(q, q, mb, nb)[1, 0])


@pytest.mark.parametrize("form", FORMS)
def test_fp32_random_ragged(form):
    q, (mb, kp, nb) = 2, (70, 33, 45)
    M, K, N = mb * q, kp * q, nb * q
    A, B = gemm_inputs(7, form, M, K, N, "fp32", "u", "n1")
    dC = _run(form, A, B, M, K, N, q, "fp32")
    _check_blocks(dC, summa.product(form, A, B), M, N, q, TOL["fp32"])


# tile variants 0-9; 1000 + v = the same tile with the other of the two k-loops the tiles that own a CU are compiled with
@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 1000, 1001, 1002, 1008, 1009])
@pytest.mark.parametrize("form", FORMS)
def test_every_tile_variant(form, variant):
    # 32 slabs of 32 per block: first cycle, steady-state cycles and last cycle of the k-loop all run
    q, mb, kp, nb = 2, 512, 512, 512
    M, K, N = mb * q, kp * q, nb * q
    A, B = gemm_inputs(55, form, M, K, N, "bf16", "n1", "n1")
    want = summa.product(form, A, B)
    try:
        opt.debug_set_gemm_variant(variant)
        dC = _run(form, A, B, M, K, N, q, "bf16")
    finally:
        opt.debug_set_gemm_variant(-1)
    _check_blocks(dC, want, M, N, q, TOL["bf16"])


@pytest.mark.parametrize("q,mb,kp,nb,with_ws", [(2, 512, 256, 768, False), (2, 256, 2048, 256, True), (4, 1024, 1024, 256, True)],
                         ids=["wide", "long_k_split", "config2_mlp_down"])
@pytest.mark.parametrize("form", FORMS)
def test_tile_variants_give_identical_bits_and_grid_equals_device(form, q, mb, kp, nb, with_ws):
    """The planner picks the panel split from one block's shape, but the tile shape for the workgroups a launch really
    has (a whole-grid launch has q*q blocks).  That keeps grid mode = device mode bit for bit because an element walks
    the same slabs in the same order whatever tile it lies in: every fast tile variant gives the same bits, and so do
    the whole-grid launch and the q*q single-device launches (which choose different tiles).  Where the whole-grid
    launch has workgroups enough without the panel split it emulates it inside each workgroup (one accumulator per
    range of slabs, the ranges' sums added in range order): third element of the plan, same bits again."""
    M, K, N = mb * q, kp * q, nb * q
    A, B = gemm_inputs(57, form, M, K, N, "bf16", "n1", "n1")
    ws = None
    if with_ws:   # the planned panel split needs its workspace: the larger of the two modes' requests
        nbytes = max(opt.summa_workspace_bytes(form, M, K, N, q, -1, -1, opt.BF16), opt.summa_workspace_bytes(form, M, K, N, q, 0, 1, opt.BF16))
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda:0")
    ref = None
    plans = set()
    by_split = {}
    if not with_ws:   # (a forced variant plans its own panel split: the variants that plan the same one are compared)
        try:
            for variant in (0, 1, 2, 3, 6, 7, 8, 9, 1000, 1001, 1002, 1008, 1009):   # 1000 + v: the tile's other k-loop
                opt.debug_set_gemm_variant(variant)
                dC = _run(form, A, B, M, K, N, q, "bf16")
                plan = opt.binding.debug_last_gemm_plan()
                plans.add(plan[0])
                same = by_split.setdefault(plan[1], dC)
                assert torch.equal(dC.view(torch.int16), same.view(torch.int16)), (variant, plan)
        finally:
            opt.debug_set_gemm_variant(-1)
        assert len(plans) == 8          # eight different tile shapes were really used
        print("panel splits planned by the forced variants:", sorted(by_split))
    grid = _run(form, A, B, M, K, N, q, "bf16", ws=ws)
    grid_plan = opt.binding.debug_last_gemm_plan()
    ref = by_split.get(grid_plan[1], grid)
    dev = empty(M * N, "bf16")
    dev_plans = set()
    for i in range(q):
        for j in range(q):
            _run(form, A, B, M, K, N, q, "bf16", i, j, ws=ws, out=dev)
            dev_plans.add(opt.binding.debug_last_gemm_plan())
    assert torch.equal(grid.view(torch.int16), dev.view(torch.int16)) and torch.equal(grid.view(torch.int16), ref.view(torch.int16))
    print("grid plan", grid_plan, "device plans", dev_plans)
    assert all(p[1] == grid_plan[1] for p in dev_plans)   # the same panel split in both modes
    assert all(p[2] == 0 for p in dev_plans)              # one device: the real split
    if q == 4 and form == "ab":
        assert grid_plan[1] > 1 and grid_plan[2] == 1     # 16 blocks of [1024 x 4096 x 256]: emulated in the workgroups
    if with_ws:
        # the same with the large tiles forced (each with both of its k-loops): a forced tile plans its own split, so
        # each is compared with itself: whole grid (split emulated in the workgroups where there are enough of them)
        # against the single-device launches (real split, partial tiles, combine)
        try:
            big = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")   # room for any forced tile's partial tiles
            for variant in (1, 2, 8, 1001, 1002):
                opt.debug_set_gemm_variant(variant)
                g2 = _run(form, A, B, M, K, N, q, "bf16", ws=big)
                gp = opt.binding.debug_last_gemm_plan()
                d2 = empty(M * N, "bf16")
                for i in range(q):
                    for j in range(q):
                        _run(form, A, B, M, K, N, q, "bf16", i, j, ws=big, out=d2)
                assert torch.equal(g2.view(torch.int16), d2.view(torch.int16)), (variant, gp)
                # and without any workspace: the split is emulated inside the workgroups, the bits stay
                d3 = empty(M * N, "bf16")
                _run(form, A, B, M, K, N, q, "bf16", 0, 1, out=d3)
                blk = slice(1 * (M // q) * (N // q), 2 * (M // q) * (N // q))
                assert torch.equal(d3.view(torch.int16)[blk], d2.view(torch.int16)[blk]), (variant, "no workspace")
                print("forced", variant, "grid plan", gp)
        finally:
            opt.debug_set_gemm_variant(-1)


def test_closed_forms_and_identities():
    q, n = 2, 256
    I = np.eye(n, dtype=np.float32)
    B = round_to_bf16(np.random.default_rng(3).standard_normal((n, n)).astype(np.float32))
    assert np.array_equal(mat_to_host(_run("ab", I, B, n, n, n, q, "bf16"), n, n, q), B)       # I B = B exactly
    assert np.array_equal(mat_to_host(_run("abt", B, I, n, n, n, q, "bf16"), n, n, q), B)      # B I^T = B
    assert np.array_equal(mat_to_host(_run("atb", I, B, n, n, n, q, "bf16"), n, n, q), B)      # I^T B = B
    ones = np.ones((n, n), dtype=np.float32)
    assert np.all(mat_to_host(_run("ab", ones, ones, n, n, n, q, "bf16"), n, n, q) == n)
    # (A B^T)^T = B A^T
    A = round_to_bf16(np.random.default_rng(4).standard_normal((n, 2 * n)).astype(np.float32))
    B2 = round_to_bf16(np.random.default_rng(5).standard_normal((n, 2 * n)).astype(np.float32))
    c1 = mat_to_host(_run("abt", A, B2, n, 2 * n, n, q, "fp32"), n, n, q)
    c2 = mat_to_host(_run("abt", B2, A, n, 2 * n, n, q, "fp32"), n, n, q)
    assert rel_frobenius(c1.T, c2) < 1e-6


def test_determinism_and_panel_split():
    """Same call twice -> same bits; the panel-split path (workspace given) matches the oracle too."""
    form, q, mb, kp, nb = "ab", 4, 128, 2048, 64
    M, K, N = mb * q, kp * q, nb * q
    A, B = gemm_inputs(9, form, M, K, N, "bf16", "n1", "n02")
    want = summa.product(form, A, B)
    c1 = to_host(_run(form, A, B, M, K, N, q, "bf16", 1, 2))
    c2 = to_host(_run(form, A, B, M, K, N, q, "bf16", 1, 2))
    assert np.array_equal(c1, c2, equal_nan=True)
    nbytes = opt.summa_workspace_bytes(form, M, K, N, q, 1, 2, opt.BF16)
    assert nbytes > 0, "this skinny shape is expected to use the panel split"
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    c3 = _run(form, A, B, M, K, N, q, "bf16", 1, 2, ws=ws)
    _check_blocks(c3, want, M, N, q, TOL["bf16"], coords={(1, 2)})
    c4 = _run(form, A, B, M, K, N, q, "bf16", 1, 2, ws=ws)
    assert np.array_equal(to_host(c3), to_host(c4), equal_nan=True)
    # a workspace that is too small is ignored (no split), never an error
    small = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    c5 = _run(form, A, B, M, K, N, q, "bf16", 1, 2, ws=small)
    assert np.array_equal(to_host(c5), c1, equal_nan=True)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_epilogue(dtype):
    """bias slice, saved pre-activation, exact GeLU, GeLU' scaling, residual, fp32 output."""
    q, mb, kp, nb = 2, 136, 72, 200
    M, K, N = mb * q, kp * q, nb * q
    rng = np.random.default_rng(21)
    rnd = round_to_bf16 if dtype == "bf16" else (lambda x: x.astype(np.float32))
    A, B = gemm_inputs(22, "ab", M, K, N, dtype, "n1", "n1")
    A = rnd(A * 0.1)
    bias = rnd(rng.standard_normal(N).astype(np.float32))
    res = rnd(rng.standard_normal((M, N)).astype(np.float32))
    zsrc = rnd(rng.standard_normal((M, N)).astype(np.float32))
    acc = summa.matmul_ab(A, B)
    dA, dB = mat_to_dev(A, q, dtype), mat_to_dev(B, q, dtype)
    tol = TOL[dtype] if dtype == "bf16" else 2e-5
    # bias + GeLU + residual, pre-activation saved
    dC, dPre = empty(M * N, dtype), empty(M * N, dtype)
    opt.summa_ex("ab", dA, dB, dC, M, K, N, q, -1, -1, dt(dtype), bias=vec_to_dev(bias), pre_act=dPre, act=1,
                 residual=mat_to_dev(res, q, dtype))
    torch.cuda.synchronize()
    pre = acc + bias[None, :]
    assert rel_frobenius(mat_to_host(dPre, M, N, q), pre) <= tol
    assert rel_frobenius(mat_to_host(dC, M, N, q), olayer.gelu(pre) + res) <= tol
    # GeLU' scaling (backward of the activation) on one device only
    dC2 = empty(M * N, dtype)
    opt.summa_ex("ab", dA, dB, dC2, M, K, N, q, 1, 0, dt(dtype), gelu_grad_of=mat_to_dev(zsrc, q, dtype))
    torch.cuda.synchronize()
    want = acc * olayer.gelu_grad(zsrc)
    got = to_host(dC2).reshape(q, q, mb, nb)
    assert rel_frobenius(got[1, 0], blocks.block(want, q, 1, 0)) <= tol
    assert np.all(np.isnan(got[0, 0])) and np.all(np.isnan(got[1, 1]))
    if dtype == "bf16":   # fp32 output of a bf16 product (weight gradients)
        dC3 = empty(M * N, "fp32")
        opt.summa_ex("ab", dA, dB, dC3, M, K, N, q, -1, -1, opt.BF16, out_fp32=True)
        torch.cuda.synchronize()
        assert rel_frobenius(mat_to_host(dC3, M, N, q), acc) <= 1e-5


def test_bias_grad():
    q, mb, nb = 2, 300, 136
    M, N = mb * q, nb * q
    dY = round_to_bf16(np.random.default_rng(8).standard_normal((M, N)).astype(np.float32))
    for dtype in ("bf16", "fp32"):
        d = mat_to_dev(dY, q, dtype)
        out = empty(q * q * nb, "fp32")
        opt.bias_grad(d, out, M, N, q, -1, -1, dt(dtype))
        torch.cuda.synchronize()
        got = to_host(out).reshape(q, q, nb)
        for i in range(q):
            for j in range(q):
                want = blocks.block(dY, q, i, j).astype(np.float64).sum(axis=0)
                assert rel_frobenius(got[i, j], want) <= 1e-5
        # the reduce up the column to row 0 is the sum over i of the partials = column sums of dY
        assert rel_frobenius(got.sum(axis=0).reshape(-1), dY.astype(np.float64).sum(axis=0)) <= 1e-5


def test_error_codes_enqueue_nothing():
    A = empty(64, "bf16")
    with pytest.raises(opt.OptimusError) as e:
        opt.summa_ab(A, A, A, 8, 8, 9, 2, 0, 0, opt.BF16)
    assert e.value.code == opt.ESHAPE
    with pytest.raises(opt.OptimusError) as e:
        opt.summa_ab(A, A, A, 8, 8, 8, 2, 0, 5, opt.BF16)
    assert e.value.code == opt.ECOORD
    torch.cuda.synchronize()
    assert torch.isnan(A.float()).all()


FULL = [(name, g) for name in ("config2", "config3", "config4", "config5") for g in gemm_cases(name)]


@pytest.mark.parametrize("name,g", FULL, ids=[f"{n}-{g.name}" for n, g in FULL])
def test_full_size_one_device_sampled(name, g):
    """Benchmark sizes, one device's share in the launch configuration the benchmark times (explicit (i, j),
    workspace given).  The oracle recomputes sampled output rows of the device's block one by one in fp64."""
    q = g.q
    i, j = q - 1, 1
    A, B = gemm_inputs(g.seed, g.form, g.M, g.K, g.N, g.dtype, g.dist_a, g.dist_b)
    dA, dB = mat_to_dev(A, q, "bf16"), mat_to_dev(B, q, "bf16")
    dC = torch.zeros(g.M * g.N, dtype=torch.bfloat16, device="cuda:0")
    nbytes = opt.summa_workspace_bytes(g.form, g.M, g.K, g.N, q, i, j, opt.BF16)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda:0")
    opt.summa(g.form, dA, dB, dC, g.M, g.K, g.N, q, i, j, opt.BF16, ws=ws)
    torch.cuda.synchronize()
    mb, nb = g.M // q, g.N // q
    blk = to_host(dC[(i * q + j) * mb * nb:(i * q + j + 1) * mb * nb]).reshape(mb, nb)
    rows = np.unique(np.concatenate([[0, mb - 1], np.random.default_rng(1).integers(0, mb, 30)]))
    cols = slice(j * nb, (j + 1) * nb)
    R = i * mb + rows
    a_rows = A[:, R] if g.form == "atb" else A[R, :]              # the operand slices the sampled output rows depend on
    b_cols = B[cols, :] if g.form == "abt" else B[:, cols]
    want = summa.product(g.form, a_rows, b_cols)                 # [len(rows), nb]
    for k, r in enumerate(rows):
        assert rel_frobenius(blk[r], want[k]) <= TOL["bf16"], (name, g.name, r)
    # nothing outside block (i, j) was touched
    full = dC.view(torch.int16)
    assert int(torch.count_nonzero(full[:(i * q + j) * mb * nb])) == 0
    assert int(torch.count_nonzero(full[(i * q + j + 1) * mb * nb:])) == 0
