#!/usr/bin/env python3
"""Benchmark of the full-space model sweep on one MI355X.

A step = one pass of the whole hot path (decode, features, validity, ensemble
MLP, mean, mask, top-k, and for the streamed workload the on-device chunk
merge) over the whole synthetic space, inputs resident in HBM.  Default
workload: the 2^27-configuration space with 4 networks 14-64-64-1, k = 1000
(the configuration the headline metric and target are quoted on).

Prints ONE JSON line: metric, value (swept configurations per second), ms_per_step,
config, roofline (the sweep kernel against the fp32 matrix peak, from HIP events recorded
by the library on the launch stream), other_nets, cpu_baseline (the CPU oracle on the
host cores, on a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MATRIX_TFLOPS = 157.3   # MI355X published dense fp32 matrix (= fp32 vector) peak
PEAK_BF16_MATRIX_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0
# HBM bytes per sweep launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (KiB per dispatch, scaled
# by the factors a plain 1 GiB copy gives in the same run: 2.000 and 1.000).  A constant from
# one profiling run: this script cannot read those counters; the summary of that run is the
# file named beside the figure.
TRAFFIC_SOURCE = "profiles/sweep_kernel_f32mfma_cfg3.md"
TRAFFIC_BYTES = {("cfg3", "topk", "f32-mfma"): (1943.17 * 2.0 + 3049.16) * 1024.0,
                 ("cfg3", "all", "f32-mfma"): 249334.0 * 1024.0}
CPU_THREADS_CAP = 16              # the host share that goes with one GPU on the benchmark boxes


def cpu_model_string() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, single_seconds: float = 5.0, all_seconds: float = 12.0):
    """Times the CPU oracle as it stands on the host: (1) one thread over a contiguous slice of
    up to 2^20 indices, (2) all threads (one call = one pool of threads over disjoint index
    ranges, the oracle's own partitioner) over a contiguous power-of-two slice sized from (1)
    to about all_seconds, or the whole space if that is shorter.  Slices start in the middle
    of the space (for the 2^27 spaces: the block of first-parameter digit 4, whose share of
    valid configurations, 49 %, is close to the space's 47.5 %).  Work per valid configuration
    is constant, so rates scale linearly to the full space.  Returns swept configurations per
    second of leg (2) as `value`."""
    import oracle
    sp, m = w.space, w.model
    n = sp.n_configs
    host_cpus = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = host_cpus
    threads = max(1, min(CPU_THREADS_CAP, usable))
    oracle.predict_range(sp, m, 0, min(n, 256), threads=1)      # library load, page-in

    def pow2_at_most(v):
        p = 1
        while p * 2 <= v:
            p *= 2
        return p

    def timed(begin, count, nthreads):
        t0 = time.perf_counter()
        _, valid, _ = oracle.predict_range(sp, m, begin, count, threads=nthreads)
        return time.perf_counter() - t0, int(valid.sum())

    mid = n // 2
    pilot = min(n, 1 << 13)
    dt, _ = timed(mid - mid % pilot, pilot, 1)
    size1 = min(n, 1 << 20, max(pilot, pow2_at_most(int(pilot * single_seconds / max(dt, 1e-6)))))
    b1 = mid - mid % size1
    dt1, valid1 = timed(b1, size1, 1)
    est_all_rate = (size1 / dt1) * threads
    size_all = n if n / est_all_rate <= 1.5 * all_seconds else max(size1, pow2_at_most(int(est_all_rate * all_seconds)))
    size_all = min(size_all, n)
    ba = 0 if size_all == n else mid - mid % size_all
    dta, valida = timed(ba, size_all, threads)
    return {"value": size_all / dta, "unit": "configs/s", "cores": threads, "kind": "oracle",
            "sample": f"one call over the contiguous slice [{ba}, +{size_all}) of the same workload "
                      f"({valida} valid, {dta:.1f} s, {threads} threads); whole space = {n}",
            "evaluated_per_s": valida / dta,
            "single_thread": {"value": size1 / dt1, "unit": "configs/s", "evaluated_per_s": valid1 / dt1,
                              "sample": f"contiguous slice [{b1}, +{size1}) ({valid1} valid, {dt1:.1f} s)"},
            "cpu_model": cpu_model_string(), "host_logical_cpus": host_cpus, "usable_cpus": usable,
            "threads_cap": CPU_THREADS_CAP}


PEAK_FP32_VECTOR_FMA_TFLOPS = 78.6   # 256 CUs x 4 SIMDs x 16 lanes x 1 FMA x 2.4 GHz (no packed fp32)


def bench_train(args):
    """Training stage: one step = one whole training run of the paper-shaped ensemble
    (Section 5.2: 11 networks of 30 sigmoid units, each trained on 10/11 of 2000 sampled
    configurations of the convolution space) for --epochs full-batch epochs."""
    import numpy as np
    import torch
    import workloads as wl
    import paper_1506_00842_amd as T
    from paper_1506_00842_amd.api import Tuner
    from workloads.synthetic_benchmark import SyntheticBenchmark, initial_weights, parts_round_robin

    w = wl.paper_convolution()
    sp = w.space
    P, E, H, n, epochs = sp.n_params, 11, 30, args.samples, args.epochs
    eta, mu = 0.125, 0.875
    tn = Tuner(sp)
    idx_dev, found = tn.sample_valid(2015, n, 16 * n)
    assert int(found.item()) == n
    idx = idx_dev.cpu().numpy().view(np.uint32).astype(np.uint64)
    t = SyntheticBenchmark(sp, 2015).times(idx)
    parts = parts_round_robin(n, E)
    w0 = initial_weights(E, P, H, 2016)
    t_dev = torch.from_numpy(t).cuda()
    p_dev = torch.from_numpy(parts).cuda()
    w0_dev = torch.from_numpy(w0).cuda()
    w_dev = torch.empty_like(w0_dev)
    loss = torch.zeros((E, epochs + 1), dtype=torch.float32, device="cuda")
    ws = torch.empty(T.tuner_train_workspace_bytes(tn.space, n), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        T.tuner_train_ensemble(tn.space, E, H, n, idx_dev, t_dev, p_dev, w0_dev, epochs, eta, mu,
                               w_dev, loss, ws, stream, args.train_split)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    T.tuner_profile_enable(True)
    T.tuner_profile_read_train()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    train_ms, n_launch = T.tuner_profile_read_train()
    T.tuner_profile_enable(False)
    usable = (t > 0) & np.isfinite(t)
    # (network, sample) pairs a network trains on per epoch; loss evaluation of the final
    # weights is one more forward pass and is not counted
    pairs = int(sum(np.sum(usable & (parts != e)) for e in range(E)))
    # forward 2PH + 2H, backward 2PH + 7H (output error, both weight gradients, sigmoid derivative)
    flop_per_pair = 4 * P * H + 9 * H
    kernel_ms = train_ms / max(n_launch, 1)
    achieved = pairs * epochs * flop_per_pair / (kernel_ms * 1e-3) / 1e12
    l = loss.cpu().numpy()
    out = {
        "metric": "training sample-gradient evaluations per second (forward + backward + momentum update, "
                  "full-batch, 11 networks)",
        "value": pairs * epochs / (dt / args.steps), "unit": "sample-gradients/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "paper-convolution training", "n_samples": n, "usable_samples": int(usable.sum()),
                   "members": E, "hidden": H, "epochs": epochs, "learning_rate": eta, "momentum": mu,
                   "loss_first": float(l[:, 0].mean()), "loss_last": float(l[:, -1].mean()),
                   "us_per_epoch": 1e3 * kernel_ms / epochs},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_FP32_VECTOR_FMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_VECTOR_FMA_TFLOPS, "traffic": None,
                     "kernel": "train_kernel (up to 16 workgroups per network)", "kernel_ms": kernel_ms,
                     "flop_per_sample_gradient": flop_per_pair,
                     "note": "each epoch is a dependent step: latency-bound (arithmetic plus one barrier among the "
                             "network's workgroups per epoch)"},
    }
    if not args.no_cpu:
        import oracle
        ep_cpu = max(1, min(epochs, args.cpu_epochs))
        t1 = time.perf_counter()
        oracle.train_ensemble(sp, E, H, idx, t, parts, w0, ep_cpu, eta, mu)
        d1 = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": pairs * ep_cpu / d1, "unit": "sample-gradients/s", "cores": 1,
                               "kind": "oracle", "sample": f"the same training data, {ep_cpu} epochs ({d1:.1f} s)"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stage", default="sweep", choices=["sweep", "train"],
                    help="sweep: the full-space model sweep (headline); train: ensemble training")
    ap.add_argument("--samples", type=int, default=2000, help="training configurations (train stage)")
    ap.add_argument("--epochs", type=int, default=1000, help="epochs per training run (train stage)")
    ap.add_argument("--train-split", type=int, default=0,
                    help="workgroups per network (train stage; 0 = the library's choice)")
    ap.add_argument("--cpu-epochs", type=int, default=1000, help="epochs of the CPU oracle baseline (train stage)")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3",
                    help="cfg1..cfg5, cfg3-2^26, paper-convolution, paper-raycasting, paper-stereo")
    ap.add_argument("--mode", default="topk", choices=["topk", "all"])
    ap.add_argument("--net", default="f32-mfma", choices=["f32-mfma", "split16", "bf16", "valu"],
                    help="f32-mfma: fp32 matrix instructions; split16: two-plane f16 split, fp32 "
                         "accumulate (fp32 tolerance); bf16: bf16 operands (1e-2 tolerance)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (the sweep kernel's own "
                         "duration then comes from an eager pass after the timed region)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-other-nets", action="store_true",
                    help="skip the short untimed-region comparison runs of the other network evaluations")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a kernel of known HBM "
                         "traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--prepared", action="store_true",
                    help="tuner_prepare once before the warm-up, then prepared calls (no packing kernel per call)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other benchmark configurations (default workload only)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the sweep shards by index range; "
              "no multi-GPU path is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if args.stage == "train":
        return bench_train(args)

    import torch
    import workloads as wl
    import paper_1506_00842_amd as T
    from paper_1506_00842_amd.api import Sweep

    w = wl.BENCH_WORKLOADS[args.workload]()
    sp, m = w.space, w.model
    N = sp.n_configs
    chunk = w.chunk if w.chunk else N
    sw = Sweep(sp, m, w.k if args.mode == "topk" else 0, **net_kwargs(T, args.net))
    stream = torch.cuda.current_stream()
    if args.prepared:
        sw.prepare(stream)
    pred = None
    if args.mode == "all":
        pred = torch.empty(chunk, dtype=torch.float32, device=sw.device)
    step = make_step(sw, N, chunk, args.mode, pred, stream)

    if args.copy_calibration_mib:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.float32, device=sw.device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        eager_stream = stream
        side.wait_stream(eager_stream)
        gstep = make_step(sw, N, chunk, args.mode, pred, side)
        with torch.cuda.stream(side):
            gstep()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            gstep()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        T.tuner_profile_enable(True)
        T.tuner_profile_read()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
    else:
        T.tuner_profile_enable(True)
        T.tuner_profile_read()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    sweep_ms, n_launch = T.tuner_profile_read()
    T.tuner_profile_enable(False)
    # the same steps without the library's timing events (two event records per call cost a
    # few microseconds on the stream: visible on sweeps that take tens of microseconds)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay() if args.graph else step()
    torch.cuda.synchronize()
    ms_per_step_no_events = 1e3 * (time.perf_counter() - t0) / args.steps
    # spread of the kernel's duration: the same steps once more, the events read after each one
    per_step_ms = []
    T.tuner_profile_enable(True)
    for _ in range(args.steps):
        step()
        ms, nl = T.tuner_profile_read()
        if nl:
            per_step_ms.append(ms / nl)
    T.tuner_profile_enable(False)

    ms_per_step = 1e3 * dt / args.steps
    n_valid = w.n_valid if w.n_valid >= 0 else None
    roof = roofline_of(T, sw, w, args.net, sweep_ms / max(n_launch, 1), n_launch / args.steps)
    if roof is not None:
        tb = TRAFFIC_BYTES.get((args.workload, args.mode, args.net))
        roof["traffic"] = tb
        if per_step_ms:
            srt = sorted(per_step_ms)
            roof["kernel_ms_median"] = srt[len(srt) // 2] if len(srt) % 2 else 0.5 * (srt[len(srt) // 2 - 1] + srt[len(srt) // 2])
            roof["kernel_ms_min"], roof["kernel_ms_max"] = srt[0], srt[-1]
        roof["traffic_source"] = (f"{TRAFFIC_SOURCE} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, a "
                                  "constant from that profiling run, not measured by this one)") if tb else None
    out = {
        "metric": "predicted configs/sec (decode+MLP ensemble+top-k)" if args.mode == "topk"
                  else "predicted configs/sec (decode+MLP ensemble, all predictions written)",
        "value": N / (dt / args.steps), "unit": "configs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_no_events": ms_per_step_no_events,
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if args.net == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "n_configs": N, "n_valid": n_valid, "k": w.k,
                   "members": m.n_members, "widths": list(m.widths), "mode": args.mode,
                   "chunk": chunk, "net": args.net, "hip_graph": bool(args.graph), "prepared": bool(args.prepared)},
        "roofline": roof,
    }
    if args.mode == "all":
        out["hbm_write_GBs"] = 4.0 * N / (dt / args.steps) / 1e9
    if not args.no_other_nets and args.mode == "topk":
        # the same workload with the other network evaluations (3 steps each, outside the
        # timed region above): context for the choice of the matrix-core path
        others = {}
        for name in ("f32-mfma", "split16", "valu", "bf16"):
            if name == args.net:
                continue
            sw2 = Sweep(sp, m, w.k, **net_kwargs(T, name))
            r = time_steps(T, torch, make_step(sw2, N, chunk, "topk", None, stream), 3, 1)
            others[name] = {"ms_per_step": r["ms_per_step"], "configs_per_s": N / (r["ms_per_step"] * 1e-3),
                            "tolerance": 1e-2 if name == "bf16" else 1e-5}
            del sw2
        out["other_nets"] = others
    if not args.no_other_workloads and args.workload == "cfg3" and args.mode == "topk" and args.net == "f32-mfma":
        out["other_workloads"] = other_workloads(T, torch, wl, Sweep, stream)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


def net_kwargs(T, net):
    return {"f32-mfma": dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_MFMA),
            "split16": dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_SPLIT16),
            "valu": dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_VALU),
            "bf16": dict(precision=T.TUNER_BF16_MFMA, algo=T.TUNER_ALGO_AUTO)}[net]


def make_step(sw, N, chunk, mode, pred, stream):
    """One pass of the whole hot path over the whole space (in chunks with a running result
    for the streamed workload)."""
    def step():
        if mode == "topk":
            first = True
            for b in range(0, N, chunk):
                sw.topk(b, min(chunk, N - b), merge=not first, stream=stream)
                first = False
        else:
            for b in range(0, N, chunk):
                sw.predict_all(b, min(chunk, N - b), want_mask=False, out=pred, stream=stream)
    return step


def time_steps(T, torch, step, steps, warmup):
    """ms per step (host clock around `steps` steps) and the sweep kernel's own duration (HIP
    events recorded by the library on the launch stream)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    T.tuner_profile_enable(True)
    T.tuner_profile_read()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sweep_ms, n_launch = T.tuner_profile_read()
    T.tuner_profile_enable(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return {"ms_per_step": 1e3 * dt / steps, "ms_per_step_no_events": 1e3 * (time.perf_counter() - t0) / steps,
            "kernel_ms": sweep_ms / max(n_launch, 1), "launches_per_step": n_launch / steps}


def roofline_of(T, sw, w, net, kernel_ms, launches_per_step):
    """The sweep kernel against the matrix peak of its operand type.  Only arithmetic that is
    executed counts: configurations the sweep skips (invalid ones) count for nothing, and the
    layer-1 multiply-adds of the parameters that are constant over a tile of 32 configurations
    count once per tile, those read from the per-member table not at all.  The figure with
    every evaluated configuration's full network is kept as `frac_algorithmic`."""
    m = w.model
    if w.n_valid < 0 or kernel_ms <= 0:
        return None
    flop_per_cfg = 2 * m.macs_per_config
    n_hoisted = T.tuner_hoisted_parameters(sw.space, sw.model)
    executed = flop_per_cfg - 2.0 * m.n_members * m.widths[1] * n_hoisted * 31.0 / 32.0
    n_tabulated = T.tuner_tabulated_parameters(sw.space, sw.model) if net == "f32-mfma" else 0
    if n_tabulated:
        # one matrix step (2 inputs) adds the tile's vector to the table
        executed -= 2.0 * m.n_members * m.widths[1] * (n_tabulated - 2)
    peak = PEAK_BF16_MATRIX_TFLOPS if net == "bf16" else PEAK_FP32_MATRIX_TFLOPS
    bound = "mfma"
    if net == "split16":          # three f16 matrix products per fp32 product, against the f16 matrix peak
        executed *= 3.0
        peak = PEAK_BF16_MATRIX_TFLOPS
    elif net == "valu":           # plain vector FMAs, against the unpacked fp32 vector rate
        bound, peak = "alu", PEAK_FP32_VECTOR_FMA_TFLOPS
    evaluated_per_launch = w.n_valid / launches_per_step
    achieved = evaluated_per_launch * executed / (kernel_ms * 1e-3) / 1e12
    algorithmic = evaluated_per_launch * flop_per_cfg / (kernel_ms * 1e-3) / 1e12
    return {"bound": bound, "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
            "traffic": None,
            "kernel": {"f32-mfma": "sweep_kernel (fp32 MFMA 32x32x2)", "bf16": "sweep_kernel (bf16 MFMA 32x32x16)",
                       "split16": "sweep_kernel (f16 MFMA 32x32x16, two planes)", "valu": "sweep_kernel (v_fma_f32)"}[net],
            "kernel_ms": kernel_ms, "launches_per_step": launches_per_step,
            "evaluated_configs_per_launch": evaluated_per_launch,
            "executed_flop_per_config": executed, "flop_per_config": flop_per_cfg,
            "achieved_algorithmic": algorithmic, "frac_algorithmic": algorithmic / peak,
            "hoisted_parameters": n_hoisted, "tabulated_parameters": n_tabulated,
            "sigmoids_per_config": m.sigmoids_per_config}


def other_workloads(T, torch, wl, Sweep, stream):
    """The other synthetic spaces of the benchmark definition and the paper's convolution
    space, a few steps each, outside the timed region of the headline."""
    res = {}

    def leg(name, w, net, mode, steps, warmup, prepared=False):
        N = w.space.n_configs
        chunk = w.chunk if w.chunk else N
        sw = Sweep(w.space, w.model, w.k if mode == "topk" else 0, **net_kwargs(T, net))
        if prepared:
            sw.prepare(stream)
        pred = torch.empty(chunk, dtype=torch.float32, device=sw.device) if mode == "all" else None
        r = time_steps(T, torch, make_step(sw, N, chunk, mode, pred, stream), steps, warmup)
        ms = r["ms_per_step_no_events"] if r["ms_per_step"] < 1.0 else r["ms_per_step"]
        e = {"workload": w.name, "net": net, "mode": mode, "k": w.k if mode == "topk" else 0,
             "ms_per_step": ms, "configs_per_s": N / (ms * 1e-3), "sweep_kernel_ms": r["kernel_ms"],
             "launches_per_step": r["launches_per_step"], "steps": steps, "prepared": prepared}
        roof = roofline_of(T, sw, w, net, r["kernel_ms"], r["launches_per_step"])
        if roof is not None and ms >= 1.0:
            e["frac_of_peak"] = roof["frac"]
            e["peak_TFLOPs"] = roof["peak"]
            e["frac_algorithmic"] = roof["frac_algorithmic"]
        if mode == "all":
            e["hbm_write_GBs"] = 4.0 * N / (ms * 1e-3) / 1e9
        res[name] = e

    leg("cfg3-predict_all", wl.large(), "f32-mfma", "all", 5, 1)
    leg("cfg4-f32", wl.wide(), "f32-mfma", "topk", 3, 1)
    leg("cfg4-bf16", wl.wide(), "bf16", "topk", 5, 1)
    leg("cfg5-streamed-16-chunks", wl.streamed(), "f32-mfma", "topk", 2, 1)
    # short sweeps: latency per call (no roofline fraction: they are bound by fixed costs), with
    # the packing kernel in every call and with the workspace prepared once
    for prepared in (False, True):
        tag = "-prepared" if prepared else ""
        leg("cfg1-tiny" + tag, wl.tiny(), "f32-mfma", "topk", 200, 20, prepared)
        leg("cfg2-conv-shaped" + tag, wl.conv_shaped(), "f32-mfma", "topk", 200, 20, prepared)
        leg("paper-convolution" + tag, wl.paper_convolution(), "f32-mfma", "topk", 200, 20, prepared)
    return res


if __name__ == "__main__":
    main()
