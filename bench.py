#!/usr/bin/env python3
"""Benchmark of the ADPSGD hot path on one MI355X.

A step is one ADPSGD iteration over all L learners of a workload: minibatch
staging, BLSTM forward/backward of every learner, mixing and SGD update.  The
default workload is the largest model configuration ("cfg4": 16 learners,
delay-by-one, 6-layer BLSTM with 1024 cells per direction, 256-wide linear
bottleneck, 32000 classes, 128 segments x 21 frames per learner, bf16 GEMM
operands), the only one that exercises every kernel of the path.  A second,
short leg times the model-free mixing/update stress workload ("cfg5") for the
HBM part of the metric, and a third the smaller delay-by-one model ("cfg3") for
the MFMA fraction of its GEMM phases.  Inputs are seeded synthetic data, resident
in HBM before the timed region.

Prints ONE JSON line.  `roofline` describes the kernel that dominates the step
(the time-batched MFMA GEMM): algorithmic flops / its GPU time measured with HIP
events on the library's stream over the timed steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "frames/sec & learner-steps/sec (1 MI355X); mix/update HBM GB/s"
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
PEAK_HBM_GBS = 8000.0


def _config(Bd, wl, seed, variant=None):
    if wl.flat_params:
        if variant == "tri":     # the paper's ring-neighbour operator (weights 1/3); defined without stragglers
            return Bd.make_config(wl.L, wl.pattern, seed=seed, flat_params=wl.flat_params, mix=Bd.MIX_TRI)
        if variant == "sync":    # the synchronous baseline: update, then the mean of all learners
            return Bd.make_config(wl.L, Bd.SDPSGD, seed=seed, flat_params=wl.flat_params)
        return Bd.make_config(wl.L, wl.pattern, seed=seed, flat_params=wl.flat_params, straggler_p=wl.straggler_p)
    return Bd.make_config(wl.L, wl.pattern, seed=seed, input_dim=wl.input_dim, hidden=wl.hidden, layers=wl.layers,
                          bidirectional=wl.bidirectional, bottleneck=wl.bottleneck, classes=wl.classes,
                          batch=wl.batch, frames=wl.frames, precision=wl.precision)


def run_model(wl, steps, warmup, seed=0, tune=()):
    import torch
    from paper_2110_11199_amd import binding as Bd, synth
    eng = Bd.Adpsgd(_config(Bd, wl, seed))
    for key, value in tune:
        eng.tune(key, value)
    w0 = synth.initial_model(seed, eng.P, wl.init_scale)
    eng.set_params(-1, torch.from_numpy(w0).cuda())
    cdf = synth.zipf_cdf(wl.classes) if wl.label_dist == "zipf" else None
    batches = []
    for k in range(warmup + steps):          # a fresh minibatch per (learner, step), staged before timing
        batches.append([tuple(torch.from_numpy(a).cuda() for a in synth.batch(wl, seed, k, i, cdf))
                        for i in range(wl.L)])
    for k in range(warmup):
        eng.step(batches[k], wl.lr)
    Bd.adpsgd_set_profiling(eng.h, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        eng.step(batches[warmup + k], wl.lr)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = Bd.adpsgd_profile(eng.h)
    losses = eng.losses()
    eng.close()
    del eng
    torch.cuda.empty_cache()
    return dt, prof, float(losses.mean())


def run_model_replayed(wl, steps, seed=0, tune=()):
    """The same iterations as run_model, two of them recorded into a HIP graph once and replayed steps / 2 times
    (patterns whose schedule does not change with the iteration only).  Returns seconds for `steps` iterations."""
    import torch
    from paper_2110_11199_amd import binding as Bd, synth
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        eng = Bd.Adpsgd(_config(Bd, wl, seed))
        for key, value in tune:
            eng.tune(key, value)
        eng.set_params(-1, torch.from_numpy(synth.initial_model(seed, eng.P, wl.init_scale)).cuda())
        cdf = synth.zipf_cdf(wl.classes) if wl.label_dist == "zipf" else None
        bufs = [[tuple(torch.from_numpy(a).cuda() for a in synth.batch(wl, seed, k, i, cdf)) for i in range(wl.L)]
                for k in range(2)]
        for k in range(2):
            eng.step(bufs[k], wl.lr)
        stream.synchronize()
        eng.capture_begin()
        for k in range(2):
            eng.step(bufs[k], wl.lr)
        g = eng.capture_end()
        Bd.adpsgd_graph_replay(g)
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps // 2):
            Bd.adpsgd_graph_replay(g)
        stream.synchronize()
        dt = time.perf_counter() - t0
        Bd.adpsgd_graph_destroy(g)
        eng.close()
    del eng, bufs
    torch.cuda.empty_cache()
    return dt * steps / (2 * (steps // 2))


def run_flat(wl, steps, warmup, seed=0, variant=None):
    import torch
    from paper_2110_11199_amd import binding as Bd
    eng = Bd.Adpsgd(_config(Bd, wl, seed, variant))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    grads = []
    for i in range(wl.L):                     # x_i^0 ~ U(-0.05, 0.05) per learner, g_i ~ N(0, 1e-3^2), drawn once
        x = torch.empty(eng.P, device="cuda").uniform_(-0.05, 0.05, generator=gen)
        eng.set_params(i, x)
        grads.append(torch.empty(eng.P, device="cuda").normal_(0.0, 1e-3, generator=gen))
    del x
    for k in range(warmup):
        eng.step(grads, wl.lr)
    Bd.adpsgd_set_profiling(eng.h, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        eng.step(grads, wl.lr)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = Bd.adpsgd_profile(eng.h)
    active = sum(sum(eng.schedule(warmup + k)[2]) for k in range(steps))
    eng.close()
    del eng, grads
    torch.cuda.empty_cache()
    return dt, prof, active


def cpu_baseline(wl, seed=0, budget_s=12.0):
    """The numpy oracle, as it stands, timed on this host.  Two figures: with the threads its BLAS takes by
    itself, on whole learner minibatches of the workload until about budget_s seconds are spent; and pinned to
    one thread, on the first segments of one learner's minibatch (a bounded sample: one whole cfg4 minibatch
    takes most of a minute on one core)."""
    import numpy as np
    from paper_2110_11199_amd import synth
    from oracle import lstm
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    shape = lstm.Shape(wl.input_dim, wl.hidden, wl.layers, wl.bidirectional, wl.bottleneck, wl.classes,
                       wl.batch, wl.frames)
    w0 = synth.initial_model(seed, lstm.param_count(shape), wl.init_scale)
    cdf = synth.zipf_cdf(wl.classes) if wl.label_dist == "zipf" else None
    done, dt = 0, 0.0
    while done < wl.L and dt < budget_s:
        f, y = synth.batch(wl, seed, 0, done, cdf)
        t0 = time.perf_counter()
        lstm.loss_and_grad(shape, w0, f, y, np.float32)
        dt += time.perf_counter() - t0
        done += 1
    out = {"value": done * wl.batch * wl.frames / dt, "unit": "frames/s", "cores": int(cores), "kind": "oracle",
           "sample": "gradients of %d of the %d learner minibatches of one %s iteration (%.1f s of oracle time, BLAS on "
                     "%d threads); the mixing/update part of the oracle is elementwise and under 1%% of that"
                     % (done, wl.L, wl.name, dt, cores)}
    if threadpool_limits is not None:
        # one thread: the first nb segments of learner 0's minibatch (the segments of a minibatch are independent
        # of each other, so this is the same arithmetic per frame), sized to a few seconds
        per_frame = dt / (done * wl.batch * wl.frames) * cores           # rough single-thread cost per frame
        nb = max(1, min(wl.batch, int(6.0 / max(per_frame * wl.frames, 1e-9))))
        f, y = synth.batch(wl, seed, 0, 0, cdf)
        sub = shape._replace(batch=nb)
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            lstm.loss_and_grad(sub, w0, np.ascontiguousarray(f[:, :nb]), np.ascontiguousarray(y[:, :nb]), np.float32)
            dt1 = time.perf_counter() - t0
        out["one_thread"] = {"value": nb * wl.frames / dt1, "unit": "frames/s", "cores": 1,
                             "sample": "gradient of the first %d of the %d segments of learner 0's minibatch (%.1f s, "
                                       "BLAS pinned to one thread)" % (nb, wl.batch, dt1)}
    try:                                      # which host the figures are from
        with open("/proc/cpuinfo") as fh:
            names = [ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")]
        out["cpu_model"] = names[0] if names else None
    except OSError:
        out["cpu_model"] = None
    return out


def measured_peaks():
    """What this device attains on the two resources the kernels are bound by (probe kernels of the library):
    a register-only bf16 MFMA loop, and streaming passes with the read:write mixes of the update kernels."""
    import torch
    from paper_2110_11199_amd import binding as Bd
    st = torch.cuda.current_stream().cuda_stream

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best * 1e-3
    blocks, iters = 1024, 4000
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    t = timed(lambda: Bd.adpsgd_probe_mfma(out.data_ptr(), blocks, iters, st))
    res = {"mfma_bf16_TFLOPs": blocks * 4 * iters * 8 * 32768.0 / t / 1e12}
    elems = 135_000_000                                 # one model of the mixing/update stress workload per stream
    pitch = (elems * 4 + 255) // 256 * 256
    buf = torch.zeros(64 * pitch, dtype=torch.uint8, device="cuda")
    for name, (r, w4, w2) in (("hbm_read_GBps", (1, 0, 0)), ("hbm_copy_GBps", (1, 1, 0)),
                              ("hbm_2read_1write_GBps", (2, 1, 0)), ("hbm_2read_1write_1bf16_GBps", (2, 1, 1)),
                              ("hbm_2read_1write_x2_GBps", (4, 2, 0)), ("hbm_2read_1write_1bf16_x16_GBps", (32, 16, 16))):
        t = timed(lambda: Bd.adpsgd_probe_stream(r, w4, w2, buf.data_ptr(), pitch, elems, st), reps=3)
        res[name] = elems * (4 * r + 4 * w4 + 2 * w2) / t / 1e9
    del buf, out
    torch.cuda.empty_cache()
    res["note"] = ("probe kernels of the library: register-only v_mfma_f32_32x32x16_bf16 loop; streaming passes over "
                   "streams of 135e6 floats with the read:write mixes of the update kernels, one position of 1, 2 (x2) or 16 "
                   "(x16) learners' streams per thread (best of 3)")
    return res


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_cfg4_cfg5.txt")


def load_traffic(path=TRAFFIC_FILE):
    """HBM bytes per launch by kernel class, read from the committed counter summary (rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE, calibrated on a kernel of known size; the file states its commands).  Returns {class: bytes per
    launch} with the classes bench.py reports, a class being absent when the table holds no kernel of it."""
    rows = []
    try:
        with open(path) as fh:
            for ln in fh:
                parts = ln.rstrip().rsplit(None, 4)
                if ln.startswith("#") or len(parts) != 5 or not parts[0].startswith("adpsgd::"):
                    continue
                try:
                    rows.append((parts[0].strip(), int(parts[1]), float(parts[4]) * 1e9))
                except ValueError:
                    continue
    except OSError:
        return {}

    def mean(pred):
        sel = [(n, b) for name, n, b in rows if pred(name)]
        cnt = sum(n for n, _ in sel)
        return sum(n * b for n, b in sel) / cnt if cnt else None
    def count(pred):
        return sum(n for name, n, _ in rows if pred(name))
    # the global-mean update runs as two kernels per chunk of the index: bytes per iteration = (mean + apply) x chunks,
    # the chunks per iteration being their dispatches per softmax dispatch (one per iteration) in the profiled run
    upd = mean(lambda k: "::all_update_kernel" in k)
    b_mean, b_apply = mean(lambda k: "::all_mean_kernel" in k), mean(lambda k: "::all_apply_kernel" in k)
    its = count(lambda k: "::softmax_ce" in k)
    if upd is None and b_mean is not None and b_apply is not None and its:
        upd = (b_mean + b_apply) * count(lambda k: "::all_mean_kernel" in k) / its
    out = {"cfg4/batched_gemm": mean(lambda k: "::gemm_" in k),
           "cfg4/recurrent": mean(lambda k: "::rec_" in k),
           "cfg4/mix_update": upd,
           "cfg5/mix_update": mean(lambda k: "::pair_update_kernel" in k or "::pair_split_update_kernel" in k)}
    return {k: v for k, v in out.items() if v is not None}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--mix-steps", type=int, default=20, help="timed steps of the cfg5 mixing/update leg (0 = skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-straggler-model", action="store_true",
                    help="skip the wall-clock model of the slow-learner experiment (a few seconds)")
    ap.add_argument("--no-peaks", action="store_true", help="skip the attained-peak probes (MFMA loop, streaming mixes)")
    ap.add_argument("--tri", action="store_true", help="also time the ring-neighbour (weights 1/3) mixing kernel on the cfg5 shape")
    ap.add_argument("--sync", action="store_true", help="also time the synchronous baseline's update-then-mean kernel on the cfg5 shape")
    ap.add_argument("--cfg3-steps", type=int, default=5, help="timed steps of the cfg3 leg (0 = skip)")
    ap.add_argument("--small-steps", type=int, default=10, help="timed steps of the cfg1 and cfg2 legs (0 = skip)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY:VALUE",
                    help="forwarded to adpsgd_set_tuning of the model handles (tuning only), e.g. 0:12")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (L learners are replicas resident on one MI355X); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    from paper_2110_11199_amd import synth
    tune = [tuple(int(v) for v in t.split(":")) for t in args.tune]
    traffic = load_traffic()
    wl = synth.WORKLOADS[args.workload]
    peaks = None if args.no_peaks else measured_peaks()
    out = {"metric": METRIC, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}

    def hbm_roofline(prof, phases, kernel, workload, traffic_key=None, mix_probe=None):
        ms = sum(prof[p]["ms"] for p in phases)
        nbytes = sum(prof[p]["bytes"] for p in phases)
        launches = max(sum(prof[p]["launches"] for p in phases), 1)
        gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        r = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
             "traffic": traffic.get("%s/%s" % (workload, traffic_key)) if traffic_key else None, "kernel": kernel,
             "avg_launch_ms": ms / launches, "algorithmic_bytes_per_launch": nbytes / launches}
        if peaks and mix_probe:      # against a pure streaming pass with the same read:write mix on this device
            r["frac_of_attained"] = gbs / peaks[mix_probe]
            r["attained_peak"] = {"probe": mix_probe, "GBps": peaks[mix_probe]}
        return r

    if wl.flat_params:
        dt, prof, active = run_flat(wl, args.steps, args.warmup)
        ms = dt / args.steps * 1e3
        out.update({"value": 0.0, "ms_per_step": ms, "dtype": "f32",
                    "learner_steps_per_s": active / dt,
                    "config": {"workload": wl.name, "L": wl.L, "flat_params": wl.flat_params, "pattern": "random ring",
                               "straggler_p": wl.straggler_p, "note": "model-free: no frames"},
                    "roofline": hbm_roofline(prof, ["mix_update"], "pair_split_update_kernel", wl.name, "mix_update", "hbm_2read_1write_GBps")})
        out["mix_update_GBps"] = out["roofline"]["achieved"]
    else:
        dt, prof, loss = run_model(wl, args.steps, args.warmup, tune=tune)
        ms = dt / args.steps * 1e3
        frames = wl.L * wl.batch * wl.frames
        dtype = "bf16" if wl.precision else "f32"
        g = prof["batched_gemm"]
        tf = g["work"] / (g["ms"] * 1e-3) / 1e12 if g["ms"] > 0 else 0.0
        rec_ms = prof["recurrent_fwd"]["ms"] + prof["recurrent_bwd"]["ms"]
        rec_work = prof["recurrent_fwd"]["work"] + prof["recurrent_bwd"]["work"]
        peak = PEAK_TFLOPS[dtype]
        rec = hbm_roofline(prof, ["recurrent_fwd", "recurrent_bwd"], "rec_forward_*_kernel + rec_backward_*_kernel", wl.name, "recurrent")
        rec["mfma_TFLOPs"] = rec_work / (rec_ms * 1e-3) / 1e12 if rec_ms > 0 else 0.0
        out.update({
            "value": frames / (ms * 1e-3), "ms_per_step": ms, "dtype": dtype,
            "learner_steps_per_s": wl.L / (ms * 1e-3),
            "config": {"workload": wl.name, "L": wl.L, "pattern": ["fixed ring", "random ring", "delay-by-one"][wl.pattern],
                       "layers": wl.layers, "hidden_per_direction": wl.hidden, "bidirectional": bool(wl.bidirectional),
                       "bottleneck": wl.bottleneck, "classes": wl.classes, "input_dim": wl.input_dim,
                       "batch_per_learner": wl.batch, "frames": wl.frames, "frames_per_step": frames},
            "mean_loss_last_step": loss,
            "phases_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items()},
            "roofline": {"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak,
                         "traffic": traffic.get("%s/batched_gemm" % wl.name),
                         "traffic_source": "profiles/hbm_traffic_cfg4_cfg5.txt (rocprofv3 counter runs of this command; not "
                                           "measured in this run)",
                         "kernel": "gemm_dma_kernel (time-batched GEMMs)",
                         "launches_per_step": g["launches"] / args.steps,
                         "avg_launch_ms": g["ms"] / max(g["launches"], 1),
                         "flops_per_launch": g["work"] / max(g["launches"], 1),
                         "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1)},
            "roofline_recurrent": rec,
            "roofline_update": hbm_roofline(prof, ["mix_update"], "all_mean_kernel + all_apply_kernel (global mean) / pair_split_update_kernel", wl.name, "mix_update",
                                            "hbm_2read_1write_1bf16_x16_GBps" if wl.precision else "hbm_2read_1write_x2_GBps"),
        })
        if args.mix_steps > 0:
            w5 = synth.WORKLOADS["cfg5"]
            dt5, prof5, active5 = run_flat(w5, args.mix_steps, 2)
            r5 = hbm_roofline(prof5, ["mix_update"], "pair_split_update_kernel", "cfg5", "mix_update", "hbm_2read_1write_GBps")
            r5.update({"workload": "cfg5", "steps": args.mix_steps, "ms_per_step": dt5 / args.mix_steps * 1e3,
                       "learner_steps_per_s": active5 / dt5})
            out["mix_update"] = r5
            out["mix_update_GBps"] = r5["achieved"]
            if args.tri:
                dt6, prof6, active6 = run_flat(w5, args.mix_steps, 2, variant="tri")
                r6 = hbm_roofline(prof6, ["mix_update"], "tri_update_kernel", "cfg5", None, "hbm_2read_1write_GBps")
                r6.update({"workload": "cfg5 with ring-neighbour mixing (weights 1/3), no stragglers", "steps": args.mix_steps,
                           "ms_per_step": dt6 / args.mix_steps * 1e3, "learner_steps_per_s": active6 / dt6})
                out["mix_update_tri"] = r6
            if args.sync:
                dt7, prof7, active7 = run_flat(w5, args.mix_steps, 2, variant="sync")
                r7 = hbm_roofline(prof7, ["mix_update"], "sync_update_kernel", "cfg5", None, "hbm_2read_1write_GBps")
                r7.update({"workload": "cfg5 as the synchronous baseline (update, then the mean of all 64 learners), no stragglers",
                           "steps": args.mix_steps, "ms_per_step": dt7 / args.mix_steps * 1e3, "learner_steps_per_s": active7 / dt7})
                out["mix_update_sync"] = r7
        if args.cfg3_steps > 0 and wl.name != "cfg3":
            # the smaller delay-by-one model: its GEMM phases against the same peak (short K loops, M = 1344)
            w3 = synth.WORKLOADS["cfg3"]
            dt3, prof3, _ = run_model(w3, args.cfg3_steps, 2, tune=tune)
            g3 = prof3["batched_gemm"]
            tf3 = g3["work"] / (g3["ms"] * 1e-3) / 1e12 if g3["ms"] > 0 else 0.0
            r3ms = prof3["recurrent_fwd"]["ms"] + prof3["recurrent_bwd"]["ms"]
            r3 = hbm_roofline(prof3, ["recurrent_fwd", "recurrent_bwd"], "recurrent step kernels", "cfg3")
            r3["mfma_TFLOPs"] = (prof3["recurrent_fwd"]["work"] + prof3["recurrent_bwd"]["work"]) / (r3ms * 1e-3) / 1e12 if r3ms > 0 else 0.0
            ms3 = dt3 / args.cfg3_steps * 1e3
            out["roofline_cfg3"] = {
                "bound": "mfma", "achieved": tf3, "peak": PEAK_TFLOPS["bf16"], "unit": "TFLOP/s", "frac": tf3 / PEAK_TFLOPS["bf16"],
                "traffic": None, "kernel": "gemm_dma_kernel (time-batched GEMMs)", "workload": "cfg3", "steps": args.cfg3_steps,
                "ms_per_step": ms3, "frames_per_s": w3.L * w3.batch * w3.frames / (ms3 * 1e-3),
                "launches_per_step": g3["launches"] / args.cfg3_steps, "avg_launch_ms": g3["ms"] / max(g3["launches"], 1),
                "flops_per_launch": g3["work"] / max(g3["launches"], 1),
                "phases_ms_per_step": {k: v["ms"] / args.cfg3_steps for k, v in prof3.items()},
                "recurrent": r3,
                "update": hbm_roofline(prof3, ["mix_update"], "all_update_kernel", "cfg3", None, "hbm_2read_1write_1bf16_GBps")}
            if peaks:
                out["roofline_cfg3"]["frac_of_attained"] = tf3 / peaks["mfma_bf16_TFLOPs"]
        if args.small_steps > 0:
            # the two small fp32 configurations: a few hundred launches of microseconds each per step (launch-latency bound)
            small = {}
            for name in ("cfg1", "cfg2"):
                if name == wl.name:
                    continue
                ws = synth.WORKLOADS[name]
                dts, profs, _ = run_model(ws, args.small_steps, 2, tune=tune)
                mss = dts / args.small_steps * 1e3
                gs = profs["batched_gemm"]
                small[name] = {"ms_per_step": mss, "frames_per_s": ws.L * ws.batch * ws.frames / (mss * 1e-3),
                               "learner_steps_per_s": ws.L / (mss * 1e-3), "dtype": "f32", "steps": args.small_steps,
                               "launches_per_step": sum(v["launches"] for v in profs.values()) / args.small_steps,
                               "gemm_TFLOPs": gs["work"] / (gs["ms"] * 1e-3) / 1e12 if gs["ms"] > 0 else 0.0,
                               "gemm_frac_of_f32_peak": (gs["work"] / (gs["ms"] * 1e-3) / 1e12 / PEAK_TFLOPS["f32"]) if gs["ms"] > 0 else 0.0,
                               "phases_ms_per_step": {k: v["ms"] / args.small_steps for k, v in profs.items()}}
                # the same iterations replayed from a HIP graph (two recorded once); the random ring's schedule changes
                # every iteration, so it cannot be recorded
                if ws.pattern != 1 and ws.straggler_p == 0.0 and args.small_steps >= 2:
                    small[name]["graph_replay_ms_per_step"] = run_model_replayed(ws, args.small_steps, tune=tune) / args.small_steps * 1e3
                else:
                    small[name]["graph_replay_ms_per_step"] = None
            out["small_configs"] = small
        if peaks:
            out["measured_peaks"] = peaks
            if wl.precision:
                out["roofline"]["frac_of_attained"] = tf / peaks["mfma_bf16_TFLOPs"]
                out["roofline"]["attained_peak"] = {"probe": "mfma_bf16_TFLOPs", "TFLOPs": peaks["mfma_bf16_TFLOPs"]}
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(wl)
    if not args.no_straggler_model:
        # Section IV-D: one of 16 learners 5, 10, 100 times slower; the paper's own figures (16 V100, end-to-end epochs)
        # are quoted as context only
        from paper_2110_11199_amd import straggler_model
        out["straggler_model"] = {
            "what": "wall-clock model on one GPU: idle kernels stand for the learners' gradient computations (2 ms per "
                    "minibatch), 16 learners, model-free 4M-parameter vectors; slowdown relative to the run without a "
                    "straggler, per iteration and per epoch (a fixed number of learner minibatches, the paper's measure)",
            "measured": straggler_model.slowdown_table(),
            "paper_slowdown_per_epoch_16_V100": {"fixed_ring": {"5x": 1.1, "10x": 1.1, "100x": 1.3},
                                                 "random_ring": {"5x": 1.1, "10x": 1.1, "100x": 1.2},
                                                 "delay_by_one": {"5x": 4.1, "10x": 8.7, "100x": 91.7}}}
    if peaks and "measured_peaks" not in out:
        out["measured_peaks"] = peaks
    print(json.dumps(out))


if __name__ == "__main__":
    main()
