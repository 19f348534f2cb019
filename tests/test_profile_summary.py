"""Host logic: the script that turns rocprofv3's CSV output into the tracked summaries (synthetic CSV input)."""
import csv
import json

from paper_2104_05343_amd import profile_summary as ps

DOM = "void optimus::gemm_mfma_kernel<256, 128, 4, 2, true, false, true, true, false, 2>(optimus::KArgs)"
COPY = "__amd_rocclr_copyBuffer"


def _write(path, header, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def test_pmc_scales_by_the_copy_and_picks_the_first_product(tmp_path):
    hdr = ["Dispatch_Id", "Kernel_Name", "Grid_Size", "Counter_Name", "Counter_Value"]
    other = "void optimus::gemm_mfma_kernel<64, 64, 2, 2, true, true, true, false, false, 1>(optimus::KArgs)"
    fetch = [[1, COPY, 1024, "FETCH_SIZE", 131072.0],                 # 256 MiB read = 131072 units -> 2048 B per unit
             [2, DOM, 131072, "FETCH_SIZE", 65536.0], [3, DOM, 131072, "FETCH_SIZE", 65536.0],
             [4, other, 1048576, "FETCH_SIZE", 99999.0],
             [5, "void at::native::copy_kernel(int)", 64, "FETCH_SIZE", 7.0]]      # a torch kernel with "copy" in its name
    write = [[1, COPY, 1024, "WRITE_SIZE", 262144.0], [2, DOM, 131072, "WRITE_SIZE", 16384.0], [4, other, 1048576, "WRITE_SIZE", 1.0]]
    _write(tmp_path / "f.csv", hdr, fetch)
    _write(tmp_path / "w.csv", hdr, write)
    (tmp_path / "probe.json").write_text(json.dumps({"gemm": [{"name": "mlp_up.ab", "block": [2048, 4096, 4096], "plan": [1, 1, 0]}]}) + "\n")
    out = tmp_path / "traffic.json"
    ps.pmc(str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), str(tmp_path / "probe.json"), "config4", "abc1234", str(out))
    rec = json.loads(out.read_text())["config4"]["mlp_up.ab"]
    assert rec["fetch_bytes"] == 65536 * 2048 and rec["write_bytes"] == 16384 * 1024
    assert rec["plan"] == [1, 1, 0] and rec["commit"] == "abc1234" and "256, 128" in rec["kernel"]
    # a second workload is merged into the same file
    ps.pmc(str(tmp_path / "f.csv"), str(tmp_path / "w.csv"), str(tmp_path / "probe.json"), "config5", "abc1234", str(out))
    assert set(json.loads(out.read_text())) == {"config4", "config5"}


def test_trace_lists_kernels_and_the_dominant_product_runs(tmp_path):
    hdr = ["Kernel_Name", "Grid_Size_X", "Start_Timestamp", "End_Timestamp"]
    rows, t = [], 0
    for rep in range(2):                       # two runs of 30 back-to-back launches with another kernel in between
        for _ in range(30):
            rows.append([DOM, 131072, t, t + 60000 + 10000 * rep])
            t += 80000
        rows.append(["void optimus::ln_kernel<unsigned short, 1, false>(int)", 131072, t, t + 5000])
        t += 10000
    _write(tmp_path / "t.csv", hdr, rows)
    bench = {"metric": "m", "value": 1.0, "unit": "TFLOP/s", "ms_per_step": 0.9, "config": {"workload": "config4: one device"},
             "roofline": {"avg_us": 70.0}}
    (tmp_path / "b.json").write_text("noise\n" + json.dumps(bench) + "\n")
    (tmp_path / "traffic.json").write_text(json.dumps({"config4": {"mlp_up.ab": {"kernel": DOM.replace("void ", "").split("(")[0]}}}))
    ps.trace(str(tmp_path / "t.csv"), str(tmp_path / "b.json"), str(tmp_path / "o.md"), "rocprofv3 ... -- python3 bench.py", "title",
             str(tmp_path / "traffic.json"))
    md = (tmp_path / "o.md").read_text()
    assert "| 0 | 30 | 60.00 |" in md and "| 1 | 30 | 70.00 |" in md
    assert "ln_kernel" in md and '"avg_us": 70.0' in md and "rocprofv3 ... -- python3 bench.py" in md
