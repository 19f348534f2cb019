"""GPU: the planner's automatic choice (tile variant and panel split) for every SUMMA product of the benchmark
configurations 3-5, one device's share, is within 10 % of the fastest forced tile variant (each forced variant plans
its own split).  Guards the calibrated constants of the cost model against kernel changes."""
import pytest
import torch

import paper_2104_05343_amd as opt
from workloads import gemm_cases
from bench import event_time_ms

pytestmark = pytest.mark.gpu
FORCED = (0, 1, 2, 3, 6, 7, 8, 9)
SLACK = 1.10


@pytest.mark.parametrize("name", ["config3", "config4", "config5"])
def test_automatic_plan_is_close_to_the_best_forced_variant(name):
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(3)
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
    bad = []
    for g in gemm_cases(name):
        q = g.q
        i, j = q - 1, 1
        A = torch.randn(g.M * g.K, generator=gen, device="cuda:0").to(torch.bfloat16)
        B = (torch.randn(g.K * g.N, generator=gen, device="cuda:0") * 0.02).to(torch.bfloat16)
        C = torch.empty(g.M * g.N, device="cuda:0", dtype=torch.bfloat16)

        def run():
            opt.summa(g.form, A, B, C, g.M, g.K, g.N, q, i, j, opt.BF16, ws=ws)
        times = {}
        try:
            for v in FORCED:
                opt.debug_set_gemm_variant(v)
                run()
                torch.cuda.synchronize()
                if opt.debug_last_gemm_plan()[0] != v:
                    continue                      # the tile does not divide this block
                times[v] = (event_time_ms(run, 20), opt.debug_last_gemm_plan())
        finally:
            opt.debug_set_gemm_variant(-1)
        t_auto = min(event_time_ms(run, 20) for _ in range(2))
        plan = opt.debug_last_gemm_plan()
        best_v = min(times, key=lambda v: times[v][0])
        t_best = times[best_v][0]
        line = (f"{name} {g.name:13s} block [{g.M // q} x {g.K} x {g.N // q}]: automatic {plan} {t_auto * 1e3:6.1f} us, "
                f"best forced {times[best_v][1]} {t_best * 1e3:6.1f} us ({t_auto / t_best:.2f}x)")
        print(line, flush=True)
        if t_auto > SLACK * t_best:
            # near the limit a single timing decides nothing: time the two contenders again, keep each one's best
            for _ in range(3):
                try:
                    opt.debug_set_gemm_variant(best_v)
                    t_best = min(t_best, event_time_ms(run, 20))
                finally:
                    opt.debug_set_gemm_variant(-1)
                t_auto = min(t_auto, event_time_ms(run, 20))
            if t_auto > SLACK * t_best:
                bad.append(line + f"; again: {t_auto * 1e3:.1f} against {t_best * 1e3:.1f} us")
        del A, B, C
    assert not bad, "\n".join(bad)
