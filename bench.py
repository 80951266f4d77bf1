#!/usr/bin/env python3
"""Benchmark of the ADPSGD hot path on one MI355X.

A step is one ADPSGD iteration over all L learners of a workload: minibatch
staging, BLSTM forward/backward of every learner, mixing and SGD update.  The
default workload is the largest model configuration ("cfg4": 16 learners,
delay-by-one, 6-layer BLSTM with 1024 cells per direction, 256-wide linear
bottleneck, 32000 classes, 128 segments x 21 frames per learner, bf16 GEMM
operands), the only one that exercises every kernel of the path.  A second,
short leg times the model-free mixing/update stress workload ("cfg5") for the
HBM part of the metric.  Inputs are seeded synthetic data, resident in HBM
before the timed region.

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


def run_model(wl, steps, warmup, seed=0):
    import torch
    from paper_2110_11199_amd import binding as Bd, synth
    eng = Bd.Adpsgd(_config(Bd, wl, seed))
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
    """The numpy oracle, as it stands, on learner minibatches of the workload until about budget_s
    seconds of CPU work are spent."""
    import numpy as np
    from paper_2110_11199_amd import synth
    from oracle import lstm
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
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
    return {"value": done * wl.batch * wl.frames / dt, "unit": "frames/s", "cores": int(cores), "kind": "oracle",
            "sample": "gradients of %d of the %d learner minibatches of one %s iteration (%.1f s of oracle time); the "
                      "mixing/update part of the oracle is elementwise and under 1%% of that" % (done, wl.L, wl.name, dt)}


# HBM traffic per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), scaled by what
# the same counters read for cast_bf16_kernel, whose size is known (FETCH_SIZE reads 0.5x its bytes, WRITE_SIZE
# 1.0x): profiles/hbm_traffic_cfg4_cfg5.txt.  Keyed by workload; bytes per launch of the named kernel class.
TRAFFIC = {
    ("cfg4", "batched_gemm"): 2.78e9,     # mean over the 29 time-batched GEMM launches of one iteration
    ("cfg4", "recurrent"): 0.306e9,       # mean over 2 x 126 rec_forward_dma_kernel launches (0.220, half the learners each:
                                          # part of it is served by the memory-side cache) and 126 rec_backward_dma_kernel (0.478)
    ("cfg4", "mix_update"): 32.5e9,       # all_update_kernel with the bf16 copy written along
    ("cfg5", "mix_update"): 93.2e9,       # pair_update_kernel, mean over the profiled iterations
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--mix-steps", type=int, default=20, help="timed steps of the cfg5 mixing/update leg (0 = skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tri", action="store_true", help="also time the ring-neighbour (weights 1/3) mixing kernel on the cfg5 shape")
    ap.add_argument("--sync", action="store_true", help="also time the synchronous baseline's update-then-mean kernel on the cfg5 shape")
    ap.add_argument("--tune", type=int, default=None, help="forwarded to adpsgd_gemm_set_variant (tuning only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (L learners are replicas resident on one MI355X); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    from paper_2110_11199_amd import synth
    if args.tune is not None:
        from paper_2110_11199_amd import binding as _Bd
        _Bd.adpsgd_gemm_set_variant(args.tune)
    wl = synth.WORKLOADS[args.workload]
    out = {"metric": METRIC, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}

    def hbm_roofline(prof, phases, kernel, workload, traffic_key=None):
        ms = sum(prof[p]["ms"] for p in phases)
        nbytes = sum(prof[p]["bytes"] for p in phases)
        launches = max(sum(prof[p]["launches"] for p in phases), 1)
        gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        return {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                "traffic": TRAFFIC.get((workload, traffic_key)) if traffic_key else None, "kernel": kernel,
                "avg_launch_ms": ms / launches, "algorithmic_bytes_per_launch": nbytes / launches}

    if wl.flat_params:
        dt, prof, active = run_flat(wl, args.steps, args.warmup)
        ms = dt / args.steps * 1e3
        out.update({"value": 0.0, "ms_per_step": ms, "dtype": "f32",
                    "learner_steps_per_s": active / dt,
                    "config": {"workload": wl.name, "L": wl.L, "flat_params": wl.flat_params, "pattern": "random ring",
                               "straggler_p": wl.straggler_p, "note": "model-free: no frames"},
                    "roofline": hbm_roofline(prof, ["mix_update"], "pair_update_kernel", wl.name, "mix_update")})
        out["mix_update_GBps"] = out["roofline"]["achieved"]
    else:
        dt, prof, loss = run_model(wl, args.steps, args.warmup)
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
                         "traffic": TRAFFIC.get((wl.name, "batched_gemm")),
                         "kernel": "gemm_dma_kernel (time-batched GEMMs)",
                         "launches_per_step": g["launches"] / args.steps,
                         "avg_launch_ms": g["ms"] / max(g["launches"], 1),
                         "flops_per_launch": g["work"] / max(g["launches"], 1),
                         "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1)},
            "roofline_recurrent": rec,
            "roofline_update": hbm_roofline(prof, ["mix_update"], "all_update_kernel / pair_update_kernel", wl.name, "mix_update"),
        })
        if args.mix_steps > 0:
            w5 = synth.WORKLOADS["cfg5"]
            dt5, prof5, active5 = run_flat(w5, args.mix_steps, 2)
            r5 = hbm_roofline(prof5, ["mix_update"], "pair_update_kernel", "cfg5", "mix_update")
            r5.update({"workload": "cfg5", "steps": args.mix_steps, "ms_per_step": dt5 / args.mix_steps * 1e3,
                       "learner_steps_per_s": active5 / dt5})
            out["mix_update"] = r5
            out["mix_update_GBps"] = r5["achieved"]
            if args.tri:
                dt6, prof6, active6 = run_flat(w5, args.mix_steps, 2, variant="tri")
                r6 = hbm_roofline(prof6, ["mix_update"], "tri_update_kernel", "cfg5")
                r6.update({"workload": "cfg5 with ring-neighbour mixing (weights 1/3), no stragglers", "steps": args.mix_steps,
                           "ms_per_step": dt6 / args.mix_steps * 1e3, "learner_steps_per_s": active6 / dt6})
                out["mix_update_tri"] = r6
            if args.sync:
                dt7, prof7, active7 = run_flat(w5, args.mix_steps, 2, variant="sync")
                r7 = hbm_roofline(prof7, ["mix_update"], "sync_update_kernel", "cfg5")
                r7.update({"workload": "cfg5 as the synchronous baseline (update, then the mean of all 64 learners), no stragglers",
                           "steps": args.mix_steps, "ms_per_step": dt7 / args.mix_steps * 1e3, "learner_steps_per_s": active7 / dt7})
                out["mix_update_sync"] = r7
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
