"""Turns rocprofv3 output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2110_11199_amd.profile_tables stats   --csv s_kernel_stats.csv --bench line.json --cmd "..." --out FILE
    python -m paper_2110_11199_amd.profile_tables traffic --fetch f_counter_collection.csv --write w_counter_collection.csv
                                                          --bench line.json --cmd "..." --out FILE
    python -m paper_2110_11199_amd.profile_tables waves   --csv u_counter_collection.csv --cmd "..." --out FILE
    python -m paper_2110_11199_amd.profile_tables lds     --csv u_counter_collection.csv --cmd "..." --out FILE

--csv / --fetch / --write: files rocprofv3 wrote (--output-format csv); --bench: the JSON line bench.py printed in the
same run (stats) or in a run of the same command (traffic); --cmd: the full rocprofv3 command, copied into the header.
`traffic` writes the table bench.py reads its `traffic` figures from (profiles/hbm_traffic_cfg4_cfg5.txt): bytes per
launch = counter (KiB per dispatch) x 1024 x scale, the scale of each counter being what makes it read the known size
of cast_bf16_kernel (one read of L x P fp32, one write of L x P bf16) in the same run.
"""
import argparse
import collections
import csv
import json
import re


def short(name, width=88):
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*", "", name).replace("unsigned short", "bf16").replace("(anonymous namespace)::", "")
    return name[:width]


def load_counters(path, width):
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    ids = collections.defaultdict(set)
    with open(path) as fh:
        for r in csv.DictReader(fh):
            k = short(r["Kernel_Name"], width)
            agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
            ids[k].add(r["Dispatch_Id"])
    return agg, ids


def header(f, title, cmd, notes=()):
    f.write("# %s\n# command (MI355X box, run from /tmp with TMPDIR=/tmp):\n" % title)
    for ln in cmd.split("\\n"):
        f.write("#   %s\n" % ln.strip())
    for ln in notes:
        f.write("# %s\n" % ln)
    f.write("\n")


def cmd_stats(a):
    rows = list(csv.DictReader(open(a.csv)))
    bj = json.loads(open(a.bench).read().strip().splitlines()[-1])
    notes = ["rows = rocprofv3's kernel_stats.csv (all iterations of the run, warm-up included).",
             "bench line of the same run: %s %.2f ms/step, %.0f frames/s; HIP-event phase times per step (ms): %s"
             % (bj["config"]["workload"], bj["ms_per_step"], bj["value"],
                ", ".join("%s %.2f" % (k, v) for k, v in bj.get("phases_ms_per_step", {}).items()))]
    if "roofline" in bj and bj["roofline"].get("unit") == "TFLOP/s":
        r = bj["roofline"]
        gsum = sum(float(x["TotalDurationNs"]) for x in rows if "gemm_" in x["Name"])
        gcalls = sum(int(x["Calls"]) for x in rows if "gemm_" in x["Name"])
        notes.append("roofline of that line: time-batched GEMMs %.0f TFLOP/s (%.3f of %.0f), %.3f ms per launch by HIP events over "
                     "%.0f launches per step; rocprofv3 average over all gemm kernels below (both workloads of the run): %.3f ms (%d calls)"
                     % (r["achieved"], r["frac"], r["peak"], r["avg_launch_ms"], r["launches_per_step"],
                        gsum / max(gcalls, 1) / 1e6, gcalls))
    for key, label in (("roofline_recurrent", "recurrent steps"), ("roofline_update", "update"), ("mix_update", "cfg5 update")):
        if key in bj:
            r = bj[key]
            notes.append("%s: %.0f GB/s algorithmic (%.3f of %.0f), %.3f ms per launch" % (label, r["achieved"], r["frac"], r["peak"], r["avg_launch_ms"]))
    if "roofline_cfg3" in bj:
        r = bj["roofline_cfg3"]
        notes.append("cfg3 leg: %.2f ms/step, time-batched GEMMs %.0f TFLOP/s (%.3f)" % (r["ms_per_step"], r["achieved"], r["frac"]))
    with open(a.out, "w") as f:
        header(f, a.title or "rocprofv3 per-kernel summary of the benchmark", a.cmd, notes)
        f.write("%-90s %6s %12s %12s %12s %12s %7s\n" % ("kernel", "calls", "total_ms", "avg_us", "min_us", "max_us", "%"))
        for r in rows:
            f.write("%-90s %6d %12.3f %12.1f %12.1f %12.1f %7.2f\n" % (
                short(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3,
                float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["Percentage"])))


def cmd_traffic(a):
    def per_dispatch(path):
        agg, ids = load_counters(path, 72)
        return {k: (sum(v.values()) / len(ids[k]), len(ids[k])) for k, v in agg.items()}
    fe, wr = per_dispatch(a.fetch), per_dispatch(a.write)
    bj = json.loads(open(a.bench).read().strip().splitlines()[-1])
    cal = "adpsgd::cast_bf16_kernel"
    if cal not in fe or cal not in wr:
        raise SystemExit("no cast_bf16_kernel in the counter files: cannot calibrate")
    n = a.cal_elems
    cal_f = (n * 4 / 1024) / fe[cal][0]
    cal_w = (n * 2 / 1024) / wr[cal][0]
    with open(a.out, "w") as f:
        header(f, a.title or "HBM traffic per kernel launch from rocprofv3 counters", a.cmd, [
            "Counters are KiB per dispatch (mean over the dispatches of a kernel), one counter per run.  Calibration against a",
            "plain streaming kernel of known size in the same run, cast_bf16_kernel (reads %d fp32 = %.3f GB, writes %.3f GB):"
            % (n, n * 4 / 1e9, n * 2 / 1e9),
            "  FETCH_SIZE reads %.3f x the true KiB -> scale %.3f;  WRITE_SIZE scale %.3f." % (1 / cal_f, cal_f, cal_w),
            "bytes = counter x 1024 x scale.  bench.py reads its `traffic` figures from the rows below."])
        f.write("%-72s %5s %12s %12s %12s\n" % ("kernel", "n", "read_GB", "write_GB", "total_GB"))
        tot = cnt = 0
        for k in sorted(fe):
            if "adpsgd" not in k:
                continue
            r_gb = fe[k][0] * 1024 * cal_f / 1e9
            w_gb = wr.get(k, (0, 0))[0] * 1024 * cal_w / 1e9
            f.write("%-72s %5d %12.3f %12.3f %12.3f\n" % (k, fe[k][1], r_gb, w_gb, r_gb + w_gb))
            if "::gemm_" in k:
                tot += (r_gb + w_gb) * fe[k][1]
                cnt += fe[k][1]
        f.write("\n")
        if cnt and "roofline" in bj:
            f.write("# time-batched GEMMs: %.2f GB per launch on average over %d launches; algorithmic (each operand and the result once)\n"
                    "#   %.2f GB per launch in the cfg4 part of the run.\n" % (tot / cnt, cnt, bj["roofline"]["algorithmic_bytes_per_launch"] / 1e9))


def cmd_waves(a):
    agg, ids = load_counters(a.csv, 66)
    with open(a.out, "w") as f:
        header(f, a.title or "Where the wave cycles of the kernels go", a.cmd, [
            "Shares of SQ_WAVE_CYCLES, summed over the dispatches of a kernel: wait = SQ_WAIT_ANY (waiting on a memory or LDS",
            "counter), issue = SQ_WAIT_INST_ANY (an instruction is ready but its unit is taken: for the GEMMs the matrix pipe),",
            "active = SQ_ACTIVE_INST_ANY.  mfma = SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_WAVE_CYCLES) for the kernels with one wave",
            "per SIMD (gemm ..., 2, 2, 4, 4, ...): the share of time the matrix pipe of a SIMD is busy (the counter advances once",
            "per SIMD, the wave-cycle counter once per wave, four waves per workgroup; read it as an estimate)."])
        f.write("%-66s %5s %7s %7s %7s %7s\n" % ("kernel", "n", "wait", "issue", "active", "mfma"))
        for k in sorted(agg):
            c = agg[k]
            if "adpsgd" not in k or c["SQ_WAVE_CYCLES"] < 1e6:
                continue
            w = c["SQ_WAVE_CYCLES"]
            one = ", 2, 2, 4, 4," in k
            f.write("%-66s %5d %6.0f%% %6.0f%% %6.0f%% %7s\n" % (
                k, len(ids[k]), 100 * c["SQ_WAIT_ANY"] / w, 100 * c["SQ_WAIT_INST_ANY"] / w, 100 * c["SQ_ACTIVE_INST_ANY"] / w,
                ("%.0f%%" % (25 * c["SQ_VALU_MFMA_BUSY_CYCLES"] / w)) if one else "-"))


def cmd_lds(a):
    agg, ids = load_counters(a.csv, 72)
    with open(a.out, "w") as f:
        header(f, a.title or "LDS counters of the MFMA kernels", a.cmd, [
            "Sums over the dispatches of a kernel.  conflict = SQ_LDS_BANK_CONFLICT / SQ_ACTIVE_INST_LDS (cycles lost to bank",
            "conflicts per cycle the LDS is busy); wait = SQ_WAIT_INST_LDS / SQ_WAVE_CYCLES (share of wave cycles spent waiting",
            "for the LDS)."])
        f.write("%-72s %5s %16s %16s %9s %8s\n" % ("kernel", "n", "LDS_BANK_CONFLICT", "ACTIVE_INST_LDS", "conflict", "wait"))
        for k in sorted(agg):
            c = agg[k]
            if c["SQ_ACTIVE_INST_LDS"] < 1e6:
                continue
            f.write("%-72s %5d %16.4g %16.4g %8.2f%% %7.2f%%\n" % (
                k, len(ids[k]), c["SQ_LDS_BANK_CONFLICT"], c["SQ_ACTIVE_INST_LDS"],
                100 * c["SQ_LDS_BANK_CONFLICT"] / c["SQ_ACTIVE_INST_LDS"], 100 * c["SQ_WAIT_INST_LDS"] / max(c["SQ_WAVE_CYCLES"], 1)))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    for name, fn in (("stats", cmd_stats), ("traffic", cmd_traffic), ("waves", cmd_waves), ("lds", cmd_lds)):
        p = sub.add_parser(name)
        p.set_defaults(fn=fn)
        p.add_argument("--out", required=True)
        p.add_argument("--cmd", required=True, help="the rocprofv3 command line(s), '\\n' between several")
        p.add_argument("--title", default=None)
        if name in ("stats", "waves", "lds"):
            p.add_argument("--csv", required=True)
        if name in ("stats", "traffic"):
            p.add_argument("--bench", required=True)
        if name == "traffic":
            p.add_argument("--fetch", required=True)
            p.add_argument("--write", required=True)
            p.add_argument("--cal-elems", type=int, default=16 * 145145344,
                           help="elements cast_bf16_kernel converts in the run (learners x padded parameters)")
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
