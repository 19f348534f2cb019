#!/usr/bin/env python3
"""Benchmark of the per-device hot path (one MI355X).

A step is one pass of the whole hot path for ONE device (i, j) of the q x q grid: optimus_layer_fwd followed
by optimus_layer_bwd with explicit coordinates (block addressing, 2D LayerNorm, the twelve SUMMA products with
their epilogues, local attention forward/backward, bias and affine gradients), the other q*q-1 devices' blocks
being resident in HBM from one untimed grid-mode pass.  Inputs are already in HBM when the timed region starts.

Reported: value = SUMMA-product flops of the step / step time (the step also contains every non-GEMM row, so
this is a lower bound on kernel rate); roofline = the dominant SUMMA product alone, timed with HIP events on
the launch stream; per-GEMM and per-config TFLOP/s and % of the 2.5 PFLOP/s dense bf16 MFMA peak; achieved
GB/s of the LayerNorm and softmax kernels; and the CPU oracle timed on the host cores as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Bytes that crossed the L2 -> fabric boundary per launch of the dominant product come from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE) of `bench.py [--workload W] --pmc-probe`, each scaled by what the counter reads for a
# 256 MiB copy in the same run.  Hardware counters cannot be read from inside this script: the summary tool
# (python -m paper_2104_05343_amd.profile_summary pmc ...) writes them to this file together with the tile plan and
# the commit they were measured at, and they are reported only while the planner still picks that tile.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "dominant_product_traffic.json")


def measured_traffic(workload, product, plan):
    """(bytes per launch or None, note) for the dominant product from the tracked counter summary."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(workload, {}).get(product)
    except (OSError, ValueError):
        rec = None
    if rec is None:
        return None, "no counter summary for this workload under profiles/"
    if rec.get("plan") != plan:
        return None, f"counter summary was taken with tile plan {rec.get('plan')}, the planner now picks {plan}: re-profile"
    return int(rec["fetch_bytes"] + rec["write_bytes"]), f"rocprofv3 FETCH_SIZE/WRITE_SIZE scaled by a 256 MiB copy, measured at commit {rec.get('commit')}"


PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="config4", choices=["config2", "config4", "config5"])
    ap.add_argument("--device-coords", default="1,2", help="device (i,j) whose share is timed")
    ap.add_argument("--gemm-reps", type=int, default=50)
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-config GEMM table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="launch a 256 MiB copy, the dominant product and the bandwidth kernels a few times and exit "
                         "(the command profiled with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def capture(fn, reps):
    """Record `reps` back-to-back calls of fn() into one HIP graph (no host launch gaps between kernels).
    Returns a callable that replays it; falls back to an eager loop if capture is refused."""
    import torch
    fn()
    torch.cuda.synchronize()
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn()
        torch.cuda.synchronize()
        return g.replay, True
    except Exception as exc:  # pragma: no cover - depends on the runtime
        print(f"bench.py: graph capture refused ({exc}); timing eager launches", file=sys.stderr)

        def eager():
            for _ in range(reps):
                fn()
        return eager, False


LAUNCH_GRAPH = "HIP graph replay, 10 steps per graph"
STEPS_PER_GRAPH = 10   # a replay costs about 9 us on top of its kernels: amortised as a multi-layer model would


def time_steps(step, steps, warmup):
    """W untimed and exactly K timed calls of step(), replayed from HIP graphs of STEPS_PER_GRAPH steps each (the
    remainder from a one-step graph), between two synchronisations.  Returns (ms per step, graphed?)."""
    import torch
    run1, graphed = capture(step, 1)
    runN = capture(step, STEPS_PER_GRAPH)[0] if graphed and steps >= STEPS_PER_GRAPH else None

    def go(k):
        if runN is not None:
            for _ in range(k // STEPS_PER_GRAPH):
                runN()
            k %= STEPS_PER_GRAPH
        for _ in range(k):
            run1()
    go(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    go(steps)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, graphed


def event_time_ms(fn, reps, warm=1):
    """Average duration of fn() over `reps` back-to-back calls replayed from a HIP graph, measured with HIP events
    recorded on the stream the kernels run on (torch's current stream, which is also the launch stream)."""
    import torch
    run, _ = capture(fn, reps)
    for _ in range(warm):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def layer_gemm_list(b, s, h):
    """The twelve SUMMA products of a layer: (name, form, M, K, N) with (M, N) the logical output shape."""
    M = b * s
    return [
        ("qkv.ab", "ab", M, h, 3 * h), ("dense.ab", "ab", M, h, h), ("mlp_up.ab", "ab", M, h, 4 * h), ("mlp_down.ab", "ab", M, 4 * h, h),
        ("mlp_down.abt", "abt", M, h, 4 * h), ("mlp_down.atb", "atb", 4 * h, M, h),
        ("mlp_up.abt", "abt", M, 4 * h, h), ("mlp_up.atb", "atb", h, M, 4 * h),
        ("dense.abt", "abt", M, h, h), ("dense.atb", "atb", h, M, h),
        ("qkv.abt", "abt", M, 3 * h, h), ("qkv.atb", "atb", h, M, 3 * h),
    ]


ROTATE_BYTES = 320 << 20   # more than the 256 MB Infinity Cache


def time_gemms(opt, torch, gemms, q, i, j, reps, seed, rotating=True):
    """Time each product alone (device mode, workspace given) on device-generated N(0,1)/N(0,0.02) data:
    'us' with the same buffers every launch (warm caches), 'us_rotating' cycling through enough independent
    buffer sets that the device's panels of all sets exceed the Infinity Cache."""
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    rows = []
    for (name, form, M, K, N) in gemms:
        na = M * K
        nb = K * N

        def make():
            A = torch.randn(na, generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
            B = (torch.randn(nb, generator=gen, device="cuda:0", dtype=torch.float32) * 0.02).to(torch.bfloat16)
            C = torch.empty(M * N, device="cuda:0", dtype=torch.bfloat16)
            return A, B, C
        sets = [make()]
        nbytes = opt.summa_workspace_bytes(form, M, K, N, q, i, j, opt.BF16)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda:0")
        A, B, C = sets[0]
        ms = event_time_ms(lambda: opt.summa(form, A, B, C, M, K, N, q, i, j, opt.BF16, ws=ws), reps)
        plan = opt.debug_last_gemm_plan()
        fl = opt.gemm_flops(M, K, N, q)
        tf = fl / (ms * 1e-3) / 1e12
        row = {"name": name, "form": form, "block": [M // q, K, N // q], "panel": K // q, "us": round(ms * 1e3, 2),
               "tflops": round(tf, 1), "pct_peak": round(100 * tf / PEAK_BF16_TFLOPS, 1), "split_ws_bytes": int(nbytes),
               "plan": list(plan) if plan else None}
        if nbytes > 0:
            # the same product without workspace: the split is walked inside the workgroups, no partial tile reaches
            # memory, no combine launch, same bits -- what keeping every partial sum on the CU costs for this shape
            ms_n = event_time_ms(lambda: opt.summa(form, A, B, C, M, K, N, q, i, j, opt.BF16), reps)
            row["us_without_partials_in_memory"] = round(ms_n * 1e3, 2)
            row["plan_without_workspace"] = list(opt.debug_last_gemm_plan())
        if rotating:
            dev_ws = 2 * ((M // q) * K + K * (N // q) + (M // q) * (N // q))   # bytes one device touches per launch
            nsets = max(2, min(64, -(-ROTATE_BYTES // dev_ws)))
            while len(sets) < nsets:
                sets.append(make())
            turn = [0]

            def launch():
                a_, b_, c_ = sets[turn[0] % nsets]
                turn[0] += 1
                opt.summa(form, a_, b_, c_, M, K, N, q, i, j, opt.BF16, ws=ws)
            rr = nsets * max(1, reps // nsets)
            ms_r = event_time_ms(launch, rr)
            row["us_rotating"] = round(ms_r * 1e3, 2)
            row["rotating_sets"] = nsets
            row["tflops_rotating"] = round(fl / (ms_r * 1e-3) / 1e12, 1)
            row["pct_peak_rotating"] = round(100 * fl / (ms_r * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 1)
        rows.append(row)
        del A, B, C, ws, sets
    return rows


def time_bandwidth(opt, torch, b, s, h, n, q, i, j, reps, seed):
    """LayerNorm forward/backward and attention forward/backward of one device at a workload's block sizes, on
    standalone buffers: event time and achieved GB/s = algorithmic bytes / time (bf16: forward reads x, writes y and
    xhat; backward reads dy and xhat, writes dx; parameter-gradient column sums read dy and xhat once more)."""
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    M, H = b * s, h
    rows_b, cols_b = M // q, H // q

    def rnd(nel, scale=1.0):
        return (torch.randn(nel, generator=gen, device="cuda:0", dtype=torch.float32) * scale).to(torch.bfloat16)
    X, dY = rnd(M * H), rnd(M * H)
    Y, xhat, dX = (torch.empty(M * H, dtype=torch.bfloat16, device="cuda:0") for _ in range(3))
    gamma = torch.ones(H, dtype=torch.float32, device="cuda:0")
    beta = torch.zeros(H, dtype=torch.float32, device="cuda:0")
    rstd = torch.zeros(q * q * rows_b, dtype=torch.float32, device="cuda:0")
    stats = torch.zeros(q * q * rows_b * 2, dtype=torch.float32, device="cuda:0")
    bstats = torch.zeros(q * q * rows_b * 2, dtype=torch.float32, device="cuda:0")
    dg = torch.zeros(q * q * cols_b, dtype=torch.float32, device="cuda:0")
    db = torch.zeros(q * q * cols_b, dtype=torch.float32, device="cuda:0")
    # one grid-mode pass leaves the peers' partial statistics resident
    opt.layernorm2d(X, gamma, beta, Y, xhat, rstd, stats, M, H, q, -1, -1, 1e-5, opt.BF16)
    opt.layernorm2d_bwd(dY, xhat, rstd, gamma, None, dX, dg, db, bstats, M, H, q, -1, -1, opt.BF16)
    blk = rows_b * cols_b * 2
    out = {}

    def put(name, ms, nbytes, note):
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[name] = {"us": round(ms * 1e3, 2), "algorithmic_bytes": int(nbytes), "GBps": round(gbs, 1),
                     "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4), "block": [rows_b, cols_b], "what": note}
    ms = event_time_ms(lambda: opt.layernorm2d(X, gamma, beta, Y, xhat, rstd, stats, M, H, q, i, j, 1e-5, opt.BF16), reps)
    put("layernorm2d_fwd", ms, 3 * blk, "read x, write y and xhat (one kernel)")
    ms = event_time_ms(lambda: opt.layernorm2d_bwd(dY, xhat, rstd, gamma, None, dX, dg, db, bstats, M, H, q, i, j, opt.BF16), reps)
    put("layernorm2d_bwd", ms, 5 * blk, "dx kernel (read dy, xhat; write dx) + column-sum kernel (read dy, xhat)")
    # the same kernels over all q*q blocks in one launch: how far the kernels go when a launch is not latency-bound
    ms = event_time_ms(lambda: opt.layernorm2d(X, gamma, beta, Y, xhat, rstd, stats, M, H, q, -1, -1, 1e-5, opt.BF16), reps)
    put("layernorm2d_fwd_all_blocks", ms, 3 * blk * q * q, f"the same for all {q * q} blocks in one launch (the partial row statistics meet inside the launch)")
    ms = event_time_ms(lambda: opt.layernorm2d_bwd(dY, xhat, rstd, gamma, None, dX, None, None, bstats, M, H, q, -1, -1, opt.BF16), reps)
    put("layernorm2d_bwd_dx_all_blocks", ms, 3 * blk * q * q, f"dx for all {q * q} blocks in one launch (no parameter gradients)")
    # the row soft-max kernels of local attention alone, one device's score matrices: fp32 scores in, bf16 out
    nmat = (b // q) * (n // q)
    sc = torch.randn(nmat * s * s, generator=gen, device="cuda:0", dtype=torch.float32) * 1.6
    pr = torch.empty(nmat * s * s, dtype=torch.bfloat16, device="cuda:0")
    ds = torch.empty(nmat * s * s, dtype=torch.bfloat16, device="cuda:0")
    tri = nmat * s * (s + 1) // 2      # entries on and below the diagonal: all a causal row reads
    ms = event_time_ms(lambda: opt.softmax_rows(sc, pr, nmat, s, True), reps)
    put("softmax_fwd", ms, tri * 4 + nmat * s * s * 2,
        f"causal, {nmat} matrices [{s} x {s}]: read fp32 scores on and below the diagonal, write every bf16 probability")
    out["softmax_fwd"]["block"] = [nmat, s, s]
    ms = event_time_ms(lambda: opt.softmax_rows_bwd(sc, pr, ds, nmat, s, True), reps)
    put("softmax_bwd", ms, tri * (4 + 2) + nmat * s * s * 2,
        "causal: read fp32 dP and bf16 P on and below the diagonal, write every bf16 dS")
    out["softmax_bwd"]["block"] = [nmat, s, s]
    del sc, pr, ds
    # attention: scores fp32 scratch -> probabilities bf16
    qkv = rnd(M * 3 * H, 0.5)
    d_attn = rnd(M * H)
    probs = torch.zeros(q * q * nmat * s * s, dtype=torch.bfloat16, device="cuda:0")
    attn = torch.empty(M * H, dtype=torch.bfloat16, device="cuda:0")
    d_qkv = torch.empty(M * 3 * H, dtype=torch.bfloat16, device="cuda:0")
    aws = torch.empty(opt.attention_workspace_bytes(b, s, h, n, q), dtype=torch.uint8, device="cuda:0")
    ms = event_time_ms(lambda: opt.attention_fwd(qkv, probs, attn, b, s, h, n, q, i, j, True, opt.BF16, aws), reps)
    d = h // n
    att_flops = 2 * 2 * nmat * s * s * d   # QK^T and PV, non-causal equivalent
    out["attention_fwd"] = {"us": round(ms * 1e3, 2), "score_matrices": nmat, "s": s, "d": d, "kernels": 3,
                            "noncausal_equiv_tflops": round(att_flops / (ms * 1e-3) / 1e12, 1),
                            "causal_useful_tflops": round(att_flops / 2 / (ms * 1e-3) / 1e12, 1)}
    ms = event_time_ms(lambda: opt.attention_bwd(qkv, probs, d_attn, d_qkv, b, s, h, n, q, i, j, True, opt.BF16, aws), reps)
    out["attention_bwd"] = {"us": round(ms * 1e3, 2), "kernels": 5,
                            "noncausal_equiv_tflops": round(2 * att_flops / (ms * 1e-3) / 1e12, 1)}
    # the same attention without the [s x s] tensors (head widths 64 and 128 only)
    if d in (64, 128):
        lse = torch.empty(q * q * nmat * s, dtype=torch.float32, device="cuda:0")
        fws = torch.empty(opt.attention_fused_workspace_bytes(b, s, h, n, q), dtype=torch.uint8, device="cuda:0")
        ms = event_time_ms(lambda: opt.attention_fused_fwd(qkv, attn, lse, b, s, h, n, q, i, j, True, opt.BF16), reps)
        out["attention_fused_fwd"] = {"us": round(ms * 1e3, 2), "kernels": 1,
                                      "noncausal_equiv_tflops": round(att_flops / (ms * 1e-3) / 1e12, 1),
                                      "causal_useful_tflops": round(att_flops / 2 / (ms * 1e-3) / 1e12, 1)}
        ms = event_time_ms(lambda: opt.attention_fused_bwd(qkv, attn, lse, d_attn, d_qkv, b, s, h, n, q, i, j, True, opt.BF16,
                                                           fws), reps)
        out["attention_fused_bwd"] = {"us": round(ms * 1e3, 2), "kernels": 2,
                                      "noncausal_equiv_tflops": round(2 * att_flops / (ms * 1e-3) / 1e12, 1)}
    return out


def time_stack(opt, torch, harness, cfg, T, b, s, h, n, q, layers, reps):
    """A stack of `layers` identical layers run for the WHOLE q*q grid on the one GPU (grid mode: shared buffers
    cannot keep the peers' blocks of every layer resident), with activation checkpointing: forward keeps the layer
    inputs only, backward recomputes each layer (without its last product) before its gradients.  Timed beside the
    same layers with every tensor kept (no recomputation), and the buffer bytes of both."""
    M = b * s
    P = [opt.make_layer_params(T)] * layers          # the same (resident) parameters for every layer: timing only
    sz = opt.stack_sizes(cfg, layers)
    raw = {k: torch.empty(getattr(sz, k), dtype=torch.uint8, device="cuda:0")
           for k in ("workspace", "forward", "backward", "conjunction", "checkpoint", "param_grad")}
    buf = opt.make_stack_buffers(raw["workspace"], raw["forward"], raw["backward"], raw["conjunction"], raw["checkpoint"])
    G = [opt.layer_grads_in(cfg, raw["param_grad"])] * layers
    out_t = torch.empty(M * h, dtype=torch.bfloat16, device="cuda:0")
    dx_t = torch.empty(M * h, dtype=torch.bfloat16, device="cuda:0")
    fwd_ms = event_time_ms(lambda: opt.stack_fwd(cfg, P, T["x"], buf, out_t), reps)
    bwd_ms = event_time_ms(lambda: opt.stack_bwd(cfg, P, G, T["d_out"], buf, dx_t), reps)
    lt = opt.make_layer_tensors(T)
    ws = torch.empty(opt.layer_workspace_bytes_grid(cfg), dtype=torch.uint8, device="cuda:0")   # the stack's own size
    lf_ms = event_time_ms(lambda: opt.layer_fwd(cfg, lt, -1, -1, ws), reps)
    lb_ms = event_time_ms(lambda: opt.layer_bwd(cfg, lt, -1, -1, ws), reps)
    kept = layers * (sz.forward + M * h * 2) + sz.backward + sz.conjunction + sz.workspace + sz.param_grad
    ckpt = sz.forward + sz.backward + sz.conjunction + sz.workspace + sz.param_grad + sz.checkpoint
    return {"layers": layers, "mode": f"grid (all {q * q} devices' work on one GPU)",
            "fwd_ms": round(fwd_ms, 3), "bwd_with_recompute_ms": round(bwd_ms, 3),
            "no_checkpoint_fwd_ms": round(layers * lf_ms, 3), "no_checkpoint_bwd_ms": round(layers * lb_ms, 3),
            "bwd_over_fwd": round(bwd_ms / fwd_ms, 2),
            "buffer_bytes": {k: int(getattr(sz, k)) for k, _ in sz._fields_},
            "bytes_checkpointed_total": int(ckpt), "bytes_all_activations_kept_total": int(kept)}


def time_model_ends(opt, torch, b, s, h, q, i, j, v, reps, seed):
    """Embedding, lm-head and cross entropy of ONE device at a workload's sizes (the paper fixes no vocabulary size:
    v = 32768 here, a power of two near common sub-word vocabularies; token indices Zipf-distributed).  HBM-bound
    kernels report algorithmic bytes / time; the lm-head is the C = A B^T product [M/q x h] x [v/q x h]^T."""
    from workloads import token_inputs
    M = b * s
    rows, vb, hb = M // q, v // q, h // q
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)

    def rnd(nel, scale=1.0):
        return (torch.randn(nel, generator=gen, device="cuda:0", dtype=torch.float32) * scale).to(torch.bfloat16)
    tok_h, lab_h = token_inputs(seed, b, s, v)
    tok, lab = torch.from_numpy(tok_h).to("cuda:0"), torch.from_numpy(lab_h).to("cuda:0")
    table, x, d_x = rnd(v * h, 0.02), torch.empty(M * h, dtype=torch.bfloat16, device="cuda:0"), rnd(M * h)
    d_table = torch.empty(v * h, dtype=torch.float32, device="cuda:0")
    logits = rnd(M * v, 2.0)
    d_logits = torch.empty(M * v, dtype=torch.bfloat16, device="cuda:0")
    loss, lse = (torch.empty(q * q * rows, dtype=torch.float32, device="cuda:0") for _ in range(2))
    stats = torch.empty(q * q * rows * 2, dtype=torch.float32, device="cuda:0")
    opt.cross_entropy2d(logits, lab, loss, lse, stats, M, v, q, -1, -1, opt.BF16)   # peers' partials resident
    out = {"v": v, "device": [i, j]}

    def put(name, ms, nbytes, note):
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[name] = {"us": round(ms * 1e3, 2), "algorithmic_bytes": int(nbytes), "GBps": round(gbs, 1),
                     "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4), "what": note}
    ms = event_time_ms(lambda: opt.embedding_fwd(tok, table, x, M, v, h, q, i, j, opt.BF16), reps)
    put("embedding_fwd", ms, 2 * rows * hb * 2 + rows * 4, f"gather {rows} rows of {hb} bf16: read + write")
    ms = event_time_ms(lambda: opt.embedding_bwd(tok, d_x, d_table, M, v, h, q, 0, j, opt.BF16), reps)
    put("embedding_bwd", ms, M * hb * 2 + vb * hb * 4 + M * 4,
        f"owner (0, {j}): read all {M} token indices and the column's d_x rows that hit its {vb} table rows (at most "
        f"{M} x {hb} bf16), write its fp32 block once")
    ms = event_time_ms(lambda: opt.cross_entropy2d(logits, lab, loss, lse, stats, M, v, q, i, j, opt.BF16), reps)
    put("cross_entropy2d", ms, rows * vb * 2, f"read the [{rows} x {vb}] bf16 logits block once (one kernel in device mode)")
    ms = event_time_ms(lambda: opt.cross_entropy2d_bwd(logits, lab, lse, d_logits, 1.0 / M, M, v, q, i, j, opt.BF16), reps)
    put("cross_entropy2d_bwd", ms, 2 * rows * vb * 2, "read logits, write d_logits")
    ms = event_time_ms(lambda: opt.summa("abt", x, table, logits, M, h, v, q, i, j, opt.BF16), reps)
    fl = 2 * rows * h * vb
    out["lm_head_abt"] = {"us": round(ms * 1e3, 2), "block": [rows, h, vb], "tflops": round(fl / (ms * 1e-3) / 1e12, 1),
                          "pct_peak": round(100 * fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 1)}
    return out


def mfma_ceiling(opt, torch):
    """What the matrix cores deliver with nothing else going on: a loop of MFMA instructions only (register operands,
    no LDS, no memory) on 64 / 128 / 256 workgroups (one per CU), with all-zero and with pseudo-random bf16 operands.
    With every CU busy on operands that toggle like real data the chip's power management keeps the rate well below
    the nominal peak: that, not 2.5 PFLOP/s, is the ceiling a product kernel on such data works under."""
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda:0")
    iters = 20000
    rows = []
    for wgs in (64, 128, 256):
        for rnd in (0, 1):
            opt.debug_mfma_rate(out, wgs, 2000, rnd)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            opt.debug_mfma_rate(out, wgs, iters, rnd)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            tf = wgs * 8 * iters * 8 * 32768 / (ms * 1e-3) / 1e12
            rows.append({"workgroups": wgs, "operands": "pseudo-random bf16" if rnd else "zeros", "ms": round(ms, 3),
                         "tflops": round(tf, 1), "frac_of_2500": round(tf / PEAK_BF16_TFLOPS, 3),
                         "frac_of_these_cus_nominal": round(tf / (PEAK_BF16_TFLOPS * wgs / 256), 3)})
    return rows


def time_layer_step(opt, torch, harness, name, steps, warmup):
    """The layer step (device mode, HIP graph replay) of another configuration, timed like the main workload's:
    reported beside it so that one default run also carries the whole-step figures of the larger layers."""
    from workloads import CONFIGS, layer_inputs, bf16_bits
    cfgd = CONFIGS[name]
    shp = cfgd["layer"]
    b, s, h, n, q = shp.b, shp.s, shp.h, shp.n, shp.q
    di, dj = 1 % q, 2 % q
    inp = layer_inputs(cfgd["seed"], shp, "bf16")
    bits = {k: bf16_bits(inp[k]) for k in ("x", "w_qkv", "w_o", "w1", "w2", "d_out")}
    vecs = {k: inp[k] for k in ("ln1_g", "ln1_b", "b_qkv", "b_o", "ln2_g", "ln2_b", "b1", "b2")}
    del inp
    res = {"workload": f"{name}: one device ({di},{dj}) of a q={q} grid, layer fwd+bwd, b={b} s={s} h={h} n={n}, causal"}
    summa_flops = sum(opt.gemm_flops(M, K, N, q) for (_, _, M, K, N) in layer_gemm_list(b, s, h))
    T0 = cfg0 = None
    for fused in (False, True):
        if fused and (h // n) not in (64, 128):
            break
        cfg, T, lt, ws = harness.alloc_layer(bits, vecs, b, s, h, n, q, causal=True, fused_attention=fused, share=T0)
        T0 = T0 or T
        cfg0 = cfg0 or cfg
        opt.layer_fwd(cfg, lt, -1, -1, ws)   # untimed grid-mode pass: every peer block resident
        opt.layer_bwd(cfg, lt, -1, -1, ws)
        torch.cuda.synchronize()

        def step():
            opt.layer_fwd(cfg, lt, di, dj, ws)
            opt.layer_bwd(cfg, lt, di, dj, ws)
        ms, graphed = time_steps(step, steps, warmup)
        key = "fused_attention" if fused else "unfused_attention"
        res[key] = {"ms_per_step": round(ms, 4), "tflops": round(summa_flops / (ms * 1e-3) / 1e12, 1),
                    "pct_of_bf16_mfma_peak": round(100 * summa_flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2),
                    "launch": LAUNCH_GRAPH if graphed else "eager launches"}
        del lt, ws
        if fused:
            del T
    return res


def config4_extras(opt, torch, harness, cfg, T, b, s, h, n, q, summa_flops):
    """Whole-grid launches of five products (the kernel on all 16 devices' blocks at once) and a two-layer
    checkpointed stack at configuration 4's size (whole grid on the one GPU)."""
    res = {}
    fwd = [g for g in layer_gemm_list(b, s, h) if g[0] in ("qkv.ab", "mlp_up.ab", "mlp_down.ab", "mlp_down.abt", "mlp_up.atb")]
    rows = time_gemms(opt, torch, fwd, q, -1, -1, 6, 78, rotating=False)
    for r in rows:   # time_gemms counts one device's flops: the grid launch does q*q times as much
        r["tflops"] = round(r["tflops"] * q * q, 1)
        r["pct_peak"] = round(100 * r["tflops"] / PEAK_BF16_TFLOPS, 1)
        r["devices"] = q * q
    res["grid_launch"] = rows
    st = time_stack(opt, torch, harness, cfg, T, b, s, h, n, q, layers=2, reps=3)
    # per layer and device: forward, recomputation without the last product (a third of the forward flops), backward
    # (twice the forward): 11/3 forward passes = 11/9 of the step's product flops
    fl = 2 * q * q * summa_flops * 11 // 9
    st["summa_tflops_fwd_bwd_recompute"] = round(fl / ((st["fwd_ms"] + st["bwd_with_recompute_ms"]) * 1e-3) / 1e12, 1)
    res["stack_2_layers"] = st
    return res


def pmc_probe(opt, torch, gemm, q, i, j):
    """A 256 MiB device copy (known traffic: 256 MiB read, 256 MiB written), then the given product, then the
    LayerNorm kernels at config-4 block size, each a few times; profiled with rocprofv3 --pmc FETCH_SIZE and, in a
    second run, --pmc WRITE_SIZE.  The copy's counter reading gives the scale of the counter."""
    n = (256 << 20) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    rows = time_gemms(opt, torch, [gemm], q, i, j, 5, 7, rotating=False)
    bw = time_bandwidth(opt, torch, 8, 1024, 4096, 32, 4, 1, 2, 3, 11)
    ends = time_model_ends(opt, torch, 8, 1024, 4096, 4, 1, 2, 32768, 3, 12)
    torch.cuda.synchronize()
    print(json.dumps({"probe": "copy 268435456 B x3; product x graph replays; layernorm/attention (both forms) and the model "
                               "ends at config-4 blocks", "gemm": rows, "bandwidth": bw, "model_ends": ends}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the other q*q-1 devices' blocks are resident in HBM); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2104_05343_amd as opt
    from paper_2104_05343_amd import harness
    from workloads import CONFIGS, layer_inputs, bf16_bits

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfgd = CONFIGS[args.workload]
    shp = cfgd["layer"]
    b, s, h, n, q = shp.b, shp.s, shp.h, shp.n, shp.q
    di, dj = (int(v) for v in args.device_coords.split(","))
    di, dj = di % q, dj % q
    if args.pmc_probe:
        dom_gemm = max(layer_gemm_list(b, s, h), key=lambda g: g[2] * g[3] * g[4])
        pmc_probe(opt, torch, dom_gemm, q, di, dj)
        return

    # ---- workload: seeded synthetic inputs of the config's recipe, uploaded and packed block-major ----
    inp = layer_inputs(cfgd["seed"], shp, "bf16")
    bits = {k: bf16_bits(inp[k]) for k in ("x", "w_qkv", "w_o", "w1", "w2", "d_out")}
    vecs = {k: inp[k] for k in ("ln1_g", "ln1_b", "b_qkv", "b_o", "ln2_g", "ln2_b", "b1", "b2")}
    cfg, T, lt, ws = harness.alloc_layer(bits, vecs, b, s, h, n, q, causal=True)
    # one untimed grid-mode pass leaves every peer block resident
    opt.layer_fwd(cfg, lt, -1, -1, ws)
    opt.layer_bwd(cfg, lt, -1, -1, ws)
    torch.cuda.synchronize()

    def step():
        opt.layer_fwd(cfg, lt, di, dj, ws)
        opt.layer_bwd(cfg, lt, di, dj, ws)

    # the step is launch-bound when issued from Python (37 small kernels, two streams): replay it from a HIP graph,
    # as a training loop would; W warm-up steps, then exactly K timed steps between two synchronisations
    ms_per_step, graphed = time_steps(step, args.steps, args.warmup)

    # the same step with the attention that keeps no [s x s] tensor (cfg.fused_attention = 1), reported beside it
    fused_step = None
    if (h // n) in (64, 128):
        cfg_f, T_f, lt_f, ws_f = harness.alloc_layer(bits, vecs, b, s, h, n, q, causal=True, fused_attention=True, share=T)
        opt.layer_fwd(cfg_f, lt_f, -1, -1, ws_f)
        opt.layer_bwd(cfg_f, lt_f, -1, -1, ws_f)
        torch.cuda.synchronize()

        def step_f():
            opt.layer_fwd(cfg_f, lt_f, di, dj, ws_f)
            opt.layer_bwd(cfg_f, lt_f, di, dj, ws_f)
        ms_f, graphed_f = time_steps(step_f, args.steps, args.warmup)
        fused_step = {"ms_per_step": round(ms_f, 4),
                      "launch": LAUNCH_GRAPH if graphed_f else "eager launches",
                      "what": "same layer step with cfg.fused_attention = 1 (no probs tensor; lse saved)"}
        del T_f, lt_f, ws_f

    gemms = layer_gemm_list(b, s, h)
    summa_flops = sum(opt.gemm_flops(M, K, N, q) for (_, _, M, K, N) in gemms)
    layer_flops = opt.layer_flops(cfg, 0) + opt.layer_flops(cfg, 1)
    value = summa_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel timings with HIP events on the launch stream ----
    fwd_ms = event_time_ms(lambda: opt.layer_fwd(cfg, lt, di, dj, ws), max(5, args.steps // 2))
    bwd_ms = event_time_ms(lambda: opt.layer_bwd(cfg, lt, di, dj, ws), max(5, args.steps // 2))
    gemm_rows = time_gemms(opt, torch, gemms, q, di, dj, args.gemm_reps, cfgd["seed"])
    # dominant kernel = the product with the most flops (first of equals): the same rule picks it in --pmc-probe.
    # Its rate is taken from the launches that cycle through independent buffer sets (the device's panels of all
    # sets exceed the 256 MB Infinity Cache: what a product sees inside a step, whose tensors pass through once);
    # the warm figure (same buffers every launch) is given beside it.
    dom = max(gemm_rows, key=lambda r: r["block"][0] * r["block"][1] * r["block"][2])
    dom_flops = 2 * dom["block"][0] * dom["block"][1] * dom["block"][2]
    alg_bytes = 2 * (dom["block"][0] * dom["block"][1] + dom["block"][1] * dom["block"][2] + dom["block"][0] * dom["block"][2])
    traffic, traffic_note = measured_traffic(args.workload, dom["name"], dom["plan"])
    roofline = {"bound": "mfma", "kernel": f"gemm_mfma_kernel ({dom['name']}, block {dom['block']}, tile plan {dom['plan']})",
                "achieved": dom["tflops_rotating"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(dom["tflops_rotating"] / PEAK_BF16_TFLOPS, 4), "flops_per_launch": dom_flops,
                "avg_us": dom["us_rotating"], "cache": f"rotating over {dom['rotating_sets']} buffer sets (> 256 MB Infinity Cache)",
                "avg_us_warm": dom["us"], "frac_warm": round(dom["tflops"] / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic, "traffic_unit": "bytes per launch crossing the L2 <-> fabric boundary", "traffic_source": traffic_note,
                "algorithmic_bytes": alg_bytes}
    sum_us = sum(r["us_rotating"] for r in gemm_rows)
    gemm_only_tflops = summa_flops / (sum_us * 1e-6) / 1e12

    # bandwidth-bound kernels: at this workload's block sizes and at config 4's (4 MiB blocks)
    bw = {args.workload: time_bandwidth(opt, torch, b, s, h, n, q, di, dj, args.gemm_reps, 5)}
    if args.workload != "config4" and not args.no_sweep:
        c4 = CONFIGS["config4"]["layer"]
        bw["config4"] = time_bandwidth(opt, torch, c4.b, c4.s, c4.h, c4.n, c4.q, 1, 2, max(5, args.gemm_reps // 3), 6)

    out = {
        "metric": "per-device SUMMA GEMM TFLOP/s (AB/ABᵀ/AᵀB) and % of MI355X bf16 MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: one device ({di},{dj}) of a q={q} grid, layer fwd+bwd, b={b} s={s} h={h} n={n}, causal",
                   "q": q, "device": [di, dj], "b": b, "s": s, "h": h, "heads": n,
                   "step": "optimus_layer_fwd + optimus_layer_bwd (device mode, peers resident)",
                   "launch": LAUNCH_GRAPH if graphed else "eager launches"},
        "pct_of_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "roofline": roofline,
        "step_detail": {"summa_flops_per_step": summa_flops, "layer_flops_per_step_table1": layer_flops,
                        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
                        "sum_of_12_gemm_kernels_us_rotating": round(sum_us, 1), "gemm_only_tflops": round(gemm_only_tflops, 1),
                        "gemm_only_pct_peak": round(100 * gemm_only_tflops / PEAK_BF16_TFLOPS, 1)},
        "step_fused_attention": fused_step,
        "gemms": gemm_rows,
        "bandwidth_kernels": bw,
        "paper_context": {"training_speedup_vs_megatron_64gpu": 1.48, "inference_speedup_vs_megatron_64gpu": 1.78,
                          "hardware": "64x Quadro RTX 5000, TACC Frontera (other machine: context, not a target)"},
    }

    out["mfma_ceiling"] = mfma_ceiling(opt, torch)
    # the dominant product against what the matrix cores of THIS box sustain on toggling operands with every CU busy
    sustained = [r["tflops"] for r in out["mfma_ceiling"] if r["workgroups"] == 256 and r["operands"] != "zeros"]
    if sustained and out.get("roofline"):
        out["roofline"]["mfma_only_sustained_tflops"] = sustained[0]
        out["roofline"]["frac_of_mfma_only_sustained"] = round(out["roofline"]["achieved"] / sustained[0], 4)
    if not args.no_sweep:
        out["model_ends"] = time_model_ends(opt, torch, b, s, h, q, di, dj, 32768, args.gemm_reps, 9)
    if not args.no_sweep and args.workload == "config4":
        out.update(config4_extras(opt, torch, harness, cfg, T, b, s, h, n, q, summa_flops))
    if not args.no_sweep and args.workload == "config2":
        out["stack"] = time_stack(opt, torch, harness, cfg, T, b, s, h, n, q, layers=4, reps=max(3, args.steps // 10))
        if (h // n) in (64, 128):
            cfg_f, T_f, _, _ = harness.alloc_layer(bits, vecs, b, s, h, n, q, causal=True, fused_attention=True, share=T)
            out["stack_fused_attention"] = time_stack(opt, torch, harness, cfg_f, T_f, b, s, h, n, q, layers=4,
                                                      reps=max(3, args.steps // 10))
            del T_f
        # the same forward products launched for the whole grid at once (i = j = -1: all q*q devices' blocks)
        fwd = [g for g in gemms if g[0] in ("qkv.ab", "mlp_up.ab", "mlp_down.ab")]
        grid_rows = time_gemms(opt, torch, fwd, q, -1, -1, max(10, args.gemm_reps // 2), 77, rotating=False)
        for r in grid_rows:   # time_gemms counts one device's flops: the grid launch does q*q times as much
            r["tflops"] = round(r["tflops"] * q * q, 1)
            r["pct_peak"] = round(100 * r["tflops"] / PEAK_BF16_TFLOPS, 1)
            r["devices"] = q * q
        out["grid_launch"] = grid_rows
    if not args.no_sweep:
        # whole-step figures of the other layer configurations (the same measurement as `value`, fewer replays)
        out["other_workload_steps"] = [time_layer_step(opt, torch, harness, name, max(10, args.steps // 2), args.warmup)
                                       for name in ("config2", "config4", "config5") if name != args.workload]

    if not args.no_sweep:
        from workloads import gemm_cases
        per = {}
        for name in ("config2", "config3", "config4", "config5"):
            cases = [(g.name, g.form, g.M, g.K, g.N) for g in gemm_cases(name)]
            qq = gemm_cases(name)[0].q
            rows = time_gemms(opt, torch, cases, qq, qq - 1, 1, max(10, args.gemm_reps // 2), 1000 + qq)
            tot_fl = sum(2 * r["block"][0] * r["block"][1] * r["block"][2] for r in rows)
            tot_us = sum(r["us_rotating"] for r in rows)
            per[name] = {"q": qq, "timing": "rotating buffer sets (aggregate, best, worst); 'us'/'pct_peak' of a row = warm",
                         "aggregate_tflops": round(tot_fl / (tot_us * 1e-6) / 1e12, 1),
                         "aggregate_pct_peak": round(100 * tot_fl / (tot_us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 1),
                         "best_pct_peak": max(r["pct_peak_rotating"] for r in rows),
                         "worst_pct_peak": min(r["pct_peak_rotating"] for r in rows),
                         "split_ws_bytes_max": max(r["split_ws_bytes"] for r in rows), "gemms": rows}
        out["per_config"] = per

    if not args.no_cpu:
        # CPU oracle (fp64 numpy, as it stands) on the host cores: the whole logical problem of this workload
        # for config2; for the larger workloads a bounded sample (the forward SUMMA products of the MLP only).
        from oracle import layer as olayer, summa as osumma
        import threadpoolctl
        info = threadpoolctl.threadpool_info()
        threads = max([d.get("num_threads", 1) for d in info] + [1])
        c0 = time.perf_counter()
        reps_cpu = 0
        while True:   # bounded sample: repeat until about 10 s of host work
            if args.workload == "config2":
                fwd_o = olayer.forward(inp, b, s, n, causal=True, keep_probs=False)
                olayer.backward(inp, fwd_o, b, s, n, causal=True)
                flops_once = 3 * 2 * 12 * b * s * h * h      # SUMMA-product flops of the full logical layer, fwd + bwd
                sample = "oracle.layer forward+backward (fp64) of the whole logical config2 layer = all 16 devices' work"
            else:
                # one sequence of the workload through the whole layer, forward and backward (every operation of the
                # layer acts on rows or on whole sequences independently, so this is 1/b of the logical layer's work)
                one = dict(inp)
                one["x"], one["d_out"] = inp["x"][:s], inp["d_out"][:s]
                fwd_o = olayer.forward(one, 1, s, n, causal=True, keep_probs=False)
                olayer.backward(one, fwd_o, 1, s, n, causal=True)
                flops_once = 3 * 2 * 12 * s * h * h
                sample = (f"oracle.layer forward+backward (fp64) of ONE sequence ({s} rows) of the logical {args.workload} "
                          f"layer = 1/{b} of all {q * q} devices' work")
            reps_cpu += 1
            if time.perf_counter() - c0 >= 10.0 or reps_cpu >= 200:
                break
        cpu_flops = flops_once * reps_cpu
        sample += f", repeated {reps_cpu}x"
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": round(cpu_flops / (c1 - c0) / 1e12, 4), "unit": "TFLOP/s", "cores": threads,
                               "kind": "oracle", "sample": sample, "seconds": round(c1 - c0, 2),
                               "os_cpu_count": os.cpu_count()}
    print(json.dumps(out, ensure_ascii=False))


if __name__ == "__main__":
    main()
