"""Host logic of the product planner (no GPU: the plan is arithmetic on shapes; without a device the planner assumes
256 compute units).  The panel split is the only part of a plan that changes the bits of a result (it fixes the order
in which the panels' contributions are added), so it must be a function of ONE device's block shape alone: the same
for device mode and grid mode, with and without a co-running product, with and without workspace.  The tile may differ."""
import pytest

import paper_2104_05343_amd as opt
from bench import layer_gemm_list
from workloads import CONFIGS, gemm_cases

plan = opt.binding.debug_plan_summa


def _products():
    out = []
    for name in ("config2", "config4", "config5"):
        shp = CONFIGS[name]["layer"]
        for (g, form, M, K, N) in layer_gemm_list(shp.b, shp.s, shp.h):
            out.append((f"{name}.{g}", form, M, K, N, shp.q))
    for c in gemm_cases("config3"):
        out.append((f"config3.{c.name}", c.form, c.M, c.K, c.N, c.q))
    return out


PRODUCTS = _products()


@pytest.mark.parametrize("case", PRODUCTS, ids=[p[0] for p in PRODUCTS])
def test_panel_split_depends_on_the_block_shape_only(case):
    _, form, M, K, N, q = case
    base = plan(form, M, K, N, q, 0, 0)
    assert base[1] >= 1
    for (i, j) in ((q - 1, 1 % q), (-1, -1)):
        for corun in (0, 1, 2):
            for have_ws in (True, False):
                p = plan(form, M, K, N, q, i, j, corun, have_ws)
                assert p[1] == base[1], (i, j, corun, have_ws, p, base)
                if not have_ws and p[1] > 1:
                    assert p[2] == 1          # no workspace: the split is walked inside the workgroups
                    assert p[0] not in (0, 4)  # the 256x256 tile has no registers for a second accumulator set


def test_no_split_without_panels_and_errors():
    # q = 1: one panel, nothing to split
    assert plan("ab", 2048, 4096, 1024, 1, 0, 0)[1] == 1
    # a skinny long-K product of the 64-device grid shape splits, a square one does not
    sk = [c for c in gemm_cases("config3") if c.name == "mlp_down.ab"][0]      # block [2048 x 1536 x 384] x 8 panels
    assert plan(sk.form, sk.M, sk.K, sk.N, sk.q, 0, 0)[1] > 1
    shp = CONFIGS["config4"]["layer"]
    assert plan("ab", shp.M, shp.h, 4 * shp.h, shp.q, 1, 2)[1] == 1
    with pytest.raises(opt.OptimusError):
        plan("ab", 2048, 4096, 1000, 3, 0, 0)            # not divisible by q
    with pytest.raises(opt.OptimusError):
        plan("ab", 2048, 4096, 1024, 4, 4, 0)            # coordinate outside the grid
    with pytest.raises(opt.OptimusError):
        plan("ab", 36, 36, 36, 4, 0, 0)                  # blocks of 9: not a matrix-core shape
