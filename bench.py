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
PEAK_HBM_GBS = 8000.0
# HBM bytes per sweep launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (KiB per dispatch, scaled
# by the factors a plain 1 GiB copy gives in the same run: 2.000 and 1.000).  Not
# measurable from inside this script; the summary of those runs is kept under profiles/.
TRAFFIC_BYTES = {("cfg3", "topk", "f32-mfma"): (2111.38 * 2.0 + 4069.60) * 1024.0,
                 ("cfg3", "all", "f32-mfma"): 250350.0 * 1024.0}


def cpu_baseline(w, target_seconds: float = 12.0, blocks: int = 0):
    """Times the CPU oracle (as it stands, all host threads through its own range
    partitioner) on blocks of 4096 indices evenly spaced over the space, so that the
    sample has the workload's own valid/invalid mix.  A short pilot sizes the sample
    to about target_seconds.  Returns swept configurations per second."""
    import oracle
    sp, m = w.space, w.model
    n = sp.n_configs
    block = min(n, 1 << 12)
    n_blocks_total = n // block
    threads = min(16, os.cpu_count() or 1)
    oracle.predict_range(sp, m, 0, min(block, 256), threads=1)      # library load, page-in

    def sweep(nb):
        step = max(1, n_blocks_total // nb)
        swept = evaluated = 0
        t0 = time.perf_counter()
        for b in range(nb):
            _, valid, _ = oracle.predict_range(sp, m, (b * step) * block, block, threads=threads)
            swept += block
            evaluated += int(valid.sum())
        return swept, evaluated, time.perf_counter() - t0

    if not blocks:
        pilot = min(n_blocks_total, 64)
        _, _, dt = sweep(pilot)
        blocks = int(max(pilot, min(n_blocks_total, pilot * target_seconds / max(dt, 1e-6))))
    swept, evaluated, dt = sweep(blocks)
    return {"value": swept / dt, "unit": "configs/s", "cores": threads, "kind": "oracle",
            "sample": f"{blocks} blocks of {block} indices evenly spaced over the space "
                      f"({swept} swept, {evaluated} valid, {dt:.1f} s)",
            "evaluated_per_s": evaluated / dt}


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
    ap.add_argument("--cpu-blocks", type=int, default=0, help="blocks of 4096 indices for the CPU baseline")
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
    net_kw = {"f32-mfma": dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_MFMA),
              "split16": dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_SPLIT16),
              "valu": dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_VALU),
              "bf16": dict(precision=T.TUNER_BF16_MFMA, algo=T.TUNER_ALGO_AUTO)}[args.net]
    sw = Sweep(sp, m, w.k if args.mode == "topk" else 0, **net_kw)
    stream = torch.cuda.current_stream()
    pred = mask = None
    if args.mode == "all":
        pred = torch.empty(chunk, dtype=torch.float32, device=sw.device)

    def step():
        if args.mode == "topk":
            first = True
            for b in range(0, N, chunk):
                sw.topk(b, min(chunk, N - b), merge=not first, stream=stream)
                first = False
        else:
            for b in range(0, N, chunk):
                sw.predict_all(b, min(chunk, N - b), want_mask=False, out=pred, stream=stream)

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
        eager_stream, stream = stream, side
        side.wait_stream(eager_stream)
        with torch.cuda.stream(side):
            step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        stream = eager_stream
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

    ms_per_step = 1e3 * dt / args.steps
    n_valid = w.n_valid if w.n_valid >= 0 else None
    flop_per_cfg = 2 * m.macs_per_config
    # layer-1 share of the parameters that are constant over a tile of 32 configurations:
    # computed once per tile, i.e. 31/32 of those multiply-adds are never executed
    n_hoisted = T.tuner_hoisted_parameters(sw.space, sw.model)
    executed_flop_per_cfg = flop_per_cfg - 2.0 * m.n_members * m.widths[1] * n_hoisted * 31.0 / 32.0
    # layer-1 share of the remaining parameters read from a per-member table: no multiply-adds
    # per configuration but the one matrix step (2 inputs) that adds the tile's vector to the table
    n_tabulated = T.tuner_tabulated_parameters(sw.space, sw.model) if args.net == "f32-mfma" else 0
    if n_tabulated:
        executed_flop_per_cfg -= 2.0 * m.n_members * m.widths[1] * (n_tabulated - 2)
    launches_per_step = n_launch / args.steps
    kernel_ms = sweep_ms / max(n_launch, 1)
    roof = None
    if n_valid is not None:
        # the sweep skips tiles with no valid configuration: only evaluated
        # configurations count as algorithmic flops
        flops_per_launch = n_valid * flop_per_cfg / launches_per_step
        achieved = flops_per_launch / (kernel_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MATRIX_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MATRIX_TFLOPS,
                "traffic": TRAFFIC_BYTES.get((args.workload, args.mode, args.net)),
                "kernel": "sweep_kernel (fp32 MFMA 32x32x2)", "kernel_ms": kernel_ms,
                "launches_per_step": launches_per_step,
                "flop_per_config": flop_per_cfg, "evaluated_configs_per_launch": n_valid / launches_per_step,
                "hoisted_parameters": n_hoisted, "tabulated_parameters": n_tabulated,
                "executed_flop_per_config": executed_flop_per_cfg,
                "frac_executed": achieved * executed_flop_per_cfg / flop_per_cfg / PEAK_FP32_MATRIX_TFLOPS,
                "sigmoids_per_config": m.sigmoids_per_config}
    out = {
        "metric": "predicted configs/sec (decode+MLP ensemble+top-k)" if args.mode == "topk"
                  else "predicted configs/sec (decode+MLP ensemble, all predictions written)",
        "value": N / (dt / args.steps), "unit": "configs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_no_events": ms_per_step_no_events,
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n_configs": N, "n_valid": n_valid, "k": w.k,
                   "members": m.n_members, "widths": list(m.widths), "mode": args.mode,
                   "chunk": chunk, "net": args.net, "hip_graph": bool(args.graph)},
        "roofline": roof,
    }
    if not args.no_other_nets and args.mode == "topk":
        # the same workload with the other network evaluations (3 steps each, outside the
        # timed region above): context for the choice of the matrix-core path
        others = {}
        for name, kw in (("f32-mfma", dict(algo=T.TUNER_ALGO_MFMA)), ("split16", dict(algo=T.TUNER_ALGO_SPLIT16)),
                         ("valu", dict(algo=T.TUNER_ALGO_VALU)), ("bf16", dict(precision=T.TUNER_BF16_MFMA))):
            if name == args.net:
                continue
            sw2 = Sweep(sp, m, w.k, **kw)

            def step2():
                first = True
                for b in range(0, N, chunk):
                    sw2.topk(b, min(chunk, N - b), merge=not first, stream=stream)
                    first = False
            step2()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(3):
                step2()
            torch.cuda.synchronize()
            d2 = (time.perf_counter() - t1) / 3
            others[name] = {"ms_per_step": 1e3 * d2, "configs_per_s": N / d2,
                            "tolerance": 1e-2 if name == "bf16" else 1e-5}
            del sw2
        out["other_nets"] = others
    if args.mode == "all":
        out["hbm_write_GBs"] = 4.0 * N / (dt / args.steps) / 1e9
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, blocks=args.cpu_blocks)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
