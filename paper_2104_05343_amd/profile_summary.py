"""Turns rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

  python -m paper_2104_05343_amd.profile_summary trace  TRACE.csv BENCH.json OUT.md "COMMAND" "TITLE" TRAFFIC.json
      per-kernel table (calls, average, min, max) of a `rocprofv3 --kernel-trace` run of bench.py, the runs of
      consecutive launches of the dominant product kernel (one run = one graph replay of bench.py's per-product
      timing: first the warm replays, then the replays over rotating buffer sets), and the bench JSON (abridged).
      The dominant product's kernel is the one TRAFFIC.json (written by `pmc` below) names for the workload.

  python -m paper_2104_05343_amd.profile_summary pmc  FETCH.csv WRITE.csv PROBE.json WORKLOAD COMMIT OUT.json
      FETCH_SIZE / WRITE_SIZE per dispatch of `bench.py --workload W --pmc-probe` (two runs: one counter each),
      scaled by what the same counter reads for the 256 MiB copy at the head of the probe; merges the dominant
      product's bytes per launch, its tile plan and the commit into OUT.json (read by bench.py for
      roofline.traffic) and prints a table of every library kernel for the text summary.
"""
import collections
import csv
import json
import statistics
import sys

COPY_BYTES = 256 << 20


def _short(name):
    return name.replace("void ", "").replace("(anonymous namespace)::", "").split("(")[0]


def _last_json(path):
    lines = [x for x in open(path) if x.startswith("{")]
    return json.loads(lines[-1])


def trace(trace_csv, bench_json, out_md, cmd, title, traffic_json):
    rows = list(csv.DictReader(open(trace_csv)))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    d = _last_json(bench_json)
    per = collections.defaultdict(list)
    for r in rows:
        per[(_short(r["Kernel_Name"]), r["Grid_Size_X"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    total = sum(sum(v) for v in per.values())
    lines = [f"# {title}", "", "Command (one MI355X, from /tmp with TMPDIR=/tmp):", "", "```", cmd, "```", "",
             "## kernels of the library by total time (rocprofv3 --kernel-trace; one line per kernel and grid size)", "",
             "| kernel | grid x | calls | total ms | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|---|---|"]
    for (k, grid), v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        if "optimus::" not in k:
            continue
        lines.append(f"| `{k}` | {grid} | {len(v)} | {sum(v) / 1e6:.3f} | {statistics.mean(v) / 1e3:.2f} | {min(v) / 1e3:.2f} | "
                     f"{max(v) / 1e3:.2f} | {100 * sum(v) / total:.2f} |")
    # dominant product: the kernel the counter summary names for this workload (largest grid of that name)
    workload = d["config"]["workload"].split(":")[0]
    try:
        named = [_short(v["kernel"]) for v in json.load(open(traffic_json)).get(workload, {}).values()]
    except (OSError, ValueError):
        named = []
    gemm = {k: v for k, v in per.items() if k[0] in named and len(v) >= 20}
    if gemm:
        dom = max(gemm, key=lambda k: int(k[1]))
        runs, cur = [], []
        for r in rows:
            if _short(r["Kernel_Name"]) == dom[0] and r["Grid_Size_X"] == dom[1]:
                cur.append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
            elif cur:
                runs.append(cur)
                cur = []
        if cur:
            runs.append(cur)
        runs = [x for x in runs if len(x) >= 10]
        lines += ["", f"## dominant product kernel `{dom[0]}` (grid {dom[1]}): runs of consecutive launches", "",
                  "One run = the launches of bench.py's per-product timing that the trace shows back to back.  In order: the replays",
                  "with the same buffers (`roofline.avg_us_warm`), then the replays cycling through independent buffer sets",
                  "(`roofline.avg_us`, the figure `roofline.achieved` is computed from).  The HIP-event figures of the JSON below",
                  "also contain the few microseconds between two launches of a graph.", "",
                  "| run | launches | avg us | min us | max us |", "|---|---|---|---|---|"]
        for k, x in enumerate(runs[:12]):
            lines.append(f"| {k} | {len(x)} | {statistics.mean(x) / 1e3:.2f} | {min(x) / 1e3:.2f} | {max(x) / 1e3:.2f} |")
    keep = ("metric", "value", "unit", "ms_per_step", "config", "roofline", "step_detail", "step_fused_attention", "gemms",
            "bandwidth_kernels", "cpu_baseline")
    lines += ["", "The run also contains torch's random-number and copy kernels that build the synthetic inputs (not listed).",
              "With kernel tracing on every launch carries the profiler's overhead, so `ms_per_step` and `value` of this run are a",
              "few percent worse than those of the same command without the profiler; the per-kernel durations are what this file is for.", "",
              "## bench.py JSON line of the same run (abridged)", "", "```json",
              json.dumps({k: d[k] for k in keep if k in d}, indent=1, ensure_ascii=False), "```", ""]
    open(out_md, "w").write("\n".join(lines) + "\n")


def _counter_medians(path, counter):
    """({(kernel, grid): median counter value}, {(kernel, grid): first dispatch id}) of one counter file."""
    agg, first = collections.defaultdict(list), {}
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            k = (_short(r["Kernel_Name"]), r.get("Grid_Size", r.get("Grid_Size_X", "")))
            agg[k].append(float(r["Counter_Value"]))
            first[k] = min(first.get(k, 1 << 62), int(r["Dispatch_Id"]))
    return {k: statistics.median(v) for k, v in agg.items()}, first


def pmc(fetch_csv, write_csv, probe_json, workload, commit, out_json):
    fetch, first = _counter_medians(fetch_csv, "FETCH_SIZE")
    write, _ = _counter_medians(write_csv, "WRITE_SIZE")

    def copy_scale(table):
        c = [v for k, v in table.items() if k[0] == "__amd_rocclr_copyBuffer"]
        if not c:
            raise SystemExit("no __amd_rocclr_copyBuffer dispatch in the counter file: cannot scale the counter")
        return COPY_BYTES / max(c)       # bytes per counter unit (the probe's copy moves 256 MiB each way)
    fs, ws = copy_scale(fetch), copy_scale(write)
    probe = _last_json(probe_json)
    g = probe["gemm"][0]
    print(f"scale: FETCH_SIZE unit = {fs:.1f} B, WRITE_SIZE unit = {ws:.1f} B")
    print("| kernel | grid | FETCH_SIZE | WRITE_SIZE | read MiB | written MiB |\n|---|---|---|---|---|---|")
    dom = None
    for k in sorted(set(fetch) | set(write)):
        if "optimus::" not in k[0]:
            continue
        f, w = fetch.get(k, 0.0), write.get(k, 0.0)
        print(f"| `{k[0]}` | {k[1]} | {f:.1f} | {w:.1f} | {f * fs / 2**20:.2f} | {w * ws / 2**20:.2f} |")
        if "gemm_mfma_kernel" in k[0] and (dom is None or first[k] < first[dom]):
            dom = k      # the probe launches the dominant product before every other product
    if dom is None:
        raise SystemExit("no product kernel in the counter files")
    try:
        table = json.load(open(out_json))
    except (OSError, ValueError):
        table = {}
    table.setdefault(workload, {})[g["name"]] = {
        "kernel": dom[0], "block": g["block"], "plan": g["plan"], "fetch_bytes": int(fetch[dom] * fs),
        "write_bytes": int(write.get(dom, 0.0) * ws), "commit": commit,
        "source": "rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE on bench.py --pmc-probe, medians per dispatch, scaled by a 256 MiB copy"}
    json.dump(table, open(out_json, "w"), indent=1)
    print("wrote", out_json, table[workload][g["name"]])


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "trace" and len(sys.argv) == 8:
        trace(*sys.argv[2:8])
    elif len(sys.argv) >= 2 and sys.argv[1] == "pmc" and len(sys.argv) == 8:
        pmc(*sys.argv[2:8])
    else:
        raise SystemExit(__doc__)
