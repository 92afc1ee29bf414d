#!/usr/bin/env python3
"""Benchmark of the Gap-Aware master update on one MI355X.

A step is one master arrival: host bookkeeping plus one fused-update launch
over all N parameters (Alg. 4 + Alg. 14), with the Gap statistics (App. C.8)
taken every --diag-every arrivals.  The default workload is the
ResNet-50-sized one: N = 25,557,032 float parameters, 64 simulated workers
with Exp(1) iteration times, one precomputed float gradient buffer per
worker, paper penalty G = |diff|/C + 1.

Prints ONE JSON line: whole-job throughput in G parameter-updates/s, the
roofline of the fused-update kernel (algorithmic bytes per launch / average
launch duration measured with events on the kernel's stream) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BYTES_PER_UPDATE = {           # algorithmic bytes per parameter per arrival, fused update
    ("ga", "f32"): 36, ("ga", "bf16"): 34, ("ga_hinge", "f32"): 36, ("ga_hinge", "bf16"): 34,
    ("asgd", "f32"): 20, ("sa", "f32"): 20, ("sa_step", "f32"): 20,
    ("asgd", "bf16"): 18, ("sa", "bf16"): 18, ("sa_step", "bf16"): 18,
}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=2000)
    p.add_argument("--warmup", type=int, default=100)
    p.add_argument("--workload", default="cfg3", choices=["cfg3", "cfg5"])
    p.add_argument("--mode", default="ga", choices=["ga", "ga_hinge", "sa", "sa_step", "asgd"])
    p.add_argument("--diag-every", type=int, default=250, help="Gap statistics every this many arrivals (0: never)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--calibration-copy", action="store_true",
                   help="after the timed region run three plain device copies of N floats (known size: 4N bytes read, "
                        "4N written) so that a counter profile of this command can be scaled")
    p.add_argument("--cpu-slice", type=int, default=1 << 22, help="parameters in the CPU-oracle sample")
    p.add_argument("--cpu-steps", type=int, default=2000, help="arrivals in the CPU-oracle sample")
    return p.parse_args()


def cpu_baseline(cfg, mode, n_slice, n_steps):
    """Time the oracle, as it stands, on a contiguous slice of the workload."""
    import numpy as np

    import ga_inputs
    import oracle
    W, seed = cfg["W"], cfg["seed"]
    n_bufs = cfg["n_bufs"]
    bufs = ga_inputs.gradient_buffers(n_bufs, n_slice, seed, cfg["grad_std"])
    if cfg["grad_dtype"] == "bf16":
        bufs = oracle.bf16_to_f32(ga_inputs.f32_to_bf16_bits(bufs)).reshape(n_bufs, n_slice)
    sched = oracle.simulate_schedule(W, n_steps, ga_inputs.DIST_CODES[cfg["dist"]], cfg["sigma"], seed)
    modes = dict(ga=oracle.MODE_GA, ga_hinge=oracle.MODE_GA_HINGE, sa=oracle.MODE_SA, sa_step=oracle.MODE_SA_STEP,
                 asgd=oracle.MODE_ASGD)
    O = oracle.Master(n_slice, W, modes[mode], oracle.Hyper(cfg["eta"], cfg["gamma"]))
    O.run_buffers(sched[:8], bufs, pick_by_worker=(cfg["pick"] == "worker"))       # touch the pages
    t0 = time.perf_counter()
    O.run_buffers(sched[8:], bufs, pick_by_worker=(cfg["pick"] == "worker"))
    dt = time.perf_counter() - t0
    updates = float(n_slice) * (n_steps - 8)
    return {"value": updates / dt / 1e9, "unit": "G param-updates/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "contiguous slice of %d parameters, all %d workers, %d arrivals of the same schedule and "
                      "gradient recipe (%.1f s)" % (n_slice, W, n_steps - 8, dt)}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the master update shards by parameter range with no "
              "exchange; see DESIGN.md). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import ga_inputs
    import paper_1909_10802_amd as ga

    cfg = dict(ga_inputs.WORKLOADS[args.workload])
    N, W, seed = cfg["N"], cfg["W"], cfg["seed"]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    K, Wm = args.steps, args.warmup

    bufs = ga_inputs.device_gradient_buffers(cfg["n_bufs"], N, seed, cfg["grad_std"], cfg["grad_dtype"], dev)
    src = ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER if cfg["pick"] == "worker" else ga.GA_PICK_BY_ARRIVAL)
    sched = ga.ga_simulate_schedule(W, K + Wm + 1, ga_inputs.DIST_CODES[cfg["dist"]], cfg["sigma"], seed)
    M = ga.Master(N, W, eta=cfg["eta"], gamma=cfg["gamma"], mode=args.mode, device=dev,
                  track_gap=(args.diag_every > 0))

    M.run_schedule(sched[:Wm], src)
    if args.diag_every > 0:
        M.diagnostics(int(sched[0]))
    torch.cuda.synchronize()

    seg = args.diag_every if args.diag_every > 0 else K
    events = []
    last_diag = None
    t0 = time.perf_counter()
    done = 0
    while done < K:
        n = min(seg, K - done)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        M.run_schedule(sched[Wm + done:Wm + done + n], src)
        e1.record()
        events.append((e0, e1))
        done += n
        if args.diag_every > 0:                                    # the Gap the next arrival will meet
            last_diag = M.diagnostics(int(sched[Wm + done]))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    kernel_ms = sum(a.elapsed_time(b) for a, b in events) / K      # average per launch, on the kernel's stream
    bpu = BYTES_PER_UPDATE[(args.mode, cfg["grad_dtype"])]
    if args.mode in ("asgd", "sa", "sa_step") and args.diag_every > 0:
        bpu += 12                                                   # gap tracking: m read + write, snapshot write
    achieved = bpu * N / (kernel_ms * 1e-3) / 1e9
    theta = M.theta()
    finite = bool(torch.isfinite(theta).all().item())
    if args.calibration_copy:
        dst = torch.empty_like(bufs[0], dtype=torch.float32) if bufs[0].dtype != torch.float32 else torch.empty_like(bufs[0])
        src_t = theta if theta.numel() == dst.numel() else theta[:dst.numel()]
        for _ in range(3):
            dst.copy_(src_t)
        torch.cuda.synchronize()

    out = {
        "metric": "G param-updates/s and achieved HBM GB/s (% of peak), GA fused update",
        "value": N * K / wall / 1e9,
        "unit": "G param-updates/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d float parameters, %d workers, %s iteration times, %d %s gradient buffers "
                               "picked by %s, one fused-update launch per arrival, mode %s"
                               % (args.workload, N, W, cfg["dist"], cfg["n_bufs"], cfg["grad_dtype"], cfg["pick"],
                                  args.mode),
                   "N": N, "n_workers": W, "mode": args.mode, "grad_dtype": cfg["grad_dtype"],
                   "eta": cfg["eta"], "gamma": cfg["gamma"], "diag_every": args.diag_every, "seed": seed},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "apply_kernel", "bytes_per_update": bpu, "avg_launch_ms": kernel_ms},
        "hbm_pct_of_peak": 100.0 * achieved / HBM_PEAK_GBS,
        "theta_finite": finite,
        "mean_gap_last": None if last_diag is None else last_diag["mean_graw"] + 1.0,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.mode, args.cpu_slice, args.cpu_steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
