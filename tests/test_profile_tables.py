"""CPU: the tool that writes the summaries under profiles/ and the reader bench.py has for them.

Small hand-made rocprofv3-style CSV files go in; the tables are checked against figures worked out by hand, and
bench.load_traffic must read back what profile_tables.traffic wrote."""
import csv
import json
import subprocess
import sys

import bench

TOOL = [sys.executable, "-m", "paper_2110_11199_amd.profile_tables"]


def _counter_csv(path, rows):
    with open(path, "w", newline="") as fh:
        w = csv.writer(fh)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for r in rows:
            w.writerow(r)


def test_traffic_table_is_calibrated_on_the_cast_kernel_and_read_back_by_the_benchmark(tmp_path):
    S = 10000                              # the table prints GB with three decimals: counters of some GB
    elems = S << 20                        # the cast kernel reads S x 4 MiB and writes S x 2 MiB
    cast, gemm = "adpsgd::cast_bf16_kernel(float const*, unsigned short*, long)", "void adpsgd::gemm_dma_kernel<unsigned short, true, true, 2, 2, 4, 4, 128, 2>(adpsgd::GemmDesc)"
    pair, sm = "adpsgd::pair_split_update_kernel<64>(adpsgd::PairArgs)", "void adpsgd::softmax_ce_row_kernel<unsigned short, 16, 512>(adpsgd::SoftmaxDesc)"
    mean, apply_ = "adpsgd::all_mean_kernel(adpsgd::AllSplitArgs)", "adpsgd::all_apply_kernel(adpsgd::AllSplitArgs)"
    # FETCH_SIZE reads half the true KiB (as on the chip), WRITE_SIZE the true KiB
    fetch = [(1, cast, "FETCH_SIZE", 2048), (2, gemm, "FETCH_SIZE", 1000), (3, gemm, "FETCH_SIZE", 3000), (4, pair, "FETCH_SIZE", 500),
             (5, sm, "FETCH_SIZE", 10), (6, mean, "FETCH_SIZE", 100), (7, mean, "FETCH_SIZE", 100), (8, apply_, "FETCH_SIZE", 50), (9, apply_, "FETCH_SIZE", 50)]
    write = [(1, cast, "WRITE_SIZE", 2048), (2, gemm, "WRITE_SIZE", 100), (3, gemm, "WRITE_SIZE", 300), (4, pair, "WRITE_SIZE", 700),
             (5, sm, "WRITE_SIZE", 10), (6, mean, "WRITE_SIZE", 20), (7, mean, "WRITE_SIZE", 20), (8, apply_, "WRITE_SIZE", 80), (9, apply_, "WRITE_SIZE", 80)]
    fetch = [(a, b, c, d * S) for a, b, c, d in fetch]
    write = [(a, b, c, d * S) for a, b, c, d in write]
    _counter_csv(tmp_path / "f.csv", fetch)
    _counter_csv(tmp_path / "w.csv", write)
    (tmp_path / "line.json").write_text(json.dumps({"roofline": {"algorithmic_bytes_per_launch": 1.0e6}}) + "\n")
    out = tmp_path / "traffic.txt"
    subprocess.run(TOOL + ["traffic", "--fetch", str(tmp_path / "f.csv"), "--write", str(tmp_path / "w.csv"), "--bench",
                           str(tmp_path / "line.json"), "--cmd", "rocprofv3 ...", "--cal-elems", str(elems), "--out", str(out)], check=True)
    text = out.read_text()
    assert "scale 2.000" in text and "WRITE_SIZE scale 1.000" in text
    got = bench.load_traffic(str(out))
    kib = 1024.0 * S
    tol = 2e6                              # three decimals of a GB, summed
    assert abs(got["cfg4/batched_gemm"] - ((1000 + 3000) / 2 * 2 + (100 + 300) / 2) * kib) < tol       # mean over its two dispatches
    assert abs(got["cfg5/mix_update"] - (500 * 2 + 700) * kib) < tol
    # two-kernel global mean: (mean + apply) x chunks per iteration = their dispatches per softmax dispatch (2 here)
    assert abs(got["cfg4/mix_update"] - ((100 * 2 + 20) + (50 * 2 + 80)) * kib * 2) < 4 * tol
    assert "cfg4/recurrent" not in got       # no recurrent kernel in the table: the class is absent, not zero


def test_wave_and_lds_tables(tmp_path):
    g = "void adpsgd::gemm_dma_kernel<unsigned short, true, true, 2, 2, 4, 4, 128, 2>(adpsgd::GemmDesc)"
    rows = []
    for did in (1, 2):
        rows += [(did, g, "SQ_WAVE_CYCLES", 2e6), (did, g, "SQ_WAIT_ANY", 5e5), (did, g, "SQ_WAIT_INST_ANY", 8e5),
                 (did, g, "SQ_ACTIVE_INST_ANY", 7e5), (did, g, "SQ_VALU_MFMA_BUSY_CYCLES", 4.8e6),
                 (did, g, "SQ_LDS_BANK_CONFLICT", 1e4), (did, g, "SQ_ACTIVE_INST_LDS", 1e6), (did, g, "SQ_WAIT_INST_LDS", 2e4)]
    _counter_csv(tmp_path / "u.csv", rows)
    subprocess.run(TOOL + ["waves", "--csv", str(tmp_path / "u.csv"), "--cmd", "rocprofv3 ...", "--out", str(tmp_path / "w.txt")], check=True)
    line = [ln for ln in (tmp_path / "w.txt").read_text().splitlines() if ln.startswith("adpsgd::gemm_dma_kernel")][0]
    assert line.split()[-5:] == ["2", "25%", "40%", "35%", "60%"]      # wait, issue, active; mfma = 25 x 4.8e6 / 2e6
    subprocess.run(TOOL + ["lds", "--csv", str(tmp_path / "u.csv"), "--cmd", "rocprofv3 ...", "--out", str(tmp_path / "l.txt")], check=True)
    line = [ln for ln in (tmp_path / "l.txt").read_text().splitlines() if ln.startswith("adpsgd::gemm_dma_kernel")][0]
    assert line.split()[-2:] == ["1.00%", "1.00%"]


def test_kernel_stats_table(tmp_path):
    with open(tmp_path / "s.csv", "w", newline="") as fh:
        w = csv.writer(fh)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        w.writerow(["void adpsgd::gemm_dma_kernel<unsigned short, true, true, 2, 2, 4, 4, 128, 2>(adpsgd::GemmDesc)", 4, 4000000, 1000000, 80.0, 900000, 1100000, 1.0])
        w.writerow(["adpsgd::pair_split_update_kernel<64>(adpsgd::PairArgs)", 2, 1000000, 500000, 20.0, 400000, 600000, 1.0])
    line = {"config": {"workload": "cfg4"}, "ms_per_step": 50.0, "value": 860160.0, "phases_ms_per_step": {"batched_gemm": 25.0},
            "roofline": {"unit": "TFLOP/s", "achieved": 1100.0, "frac": 0.44, "peak": 2500.0, "avg_launch_ms": 0.9, "launches_per_step": 29.0}}
    (tmp_path / "line.json").write_text(json.dumps(line) + "\n")
    out = tmp_path / "stats.txt"
    subprocess.run(TOOL + ["stats", "--csv", str(tmp_path / "s.csv"), "--bench", str(tmp_path / "line.json"), "--cmd", "rocprofv3 ...",
                           "--out", str(out)], check=True)
    text = out.read_text()
    assert "cfg4 50.00 ms/step" in text and "1100 TFLOP/s (0.440 of 2500)" in text and "1.000 ms (4 calls)" in text
    row = [ln for ln in text.splitlines() if ln.startswith("adpsgd::pair_split_update_kernel<64>")][0].split()
    assert row[1:] == ["2", "1.000", "500.0", "400.0", "600.0", "20.00"]
