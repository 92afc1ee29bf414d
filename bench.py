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

At 25.6 M parameters most of theta, v and m (306 MB) is served by the 256 MiB
memory-side cache, so the default run adds a second, shorter leg of the same
kernel where the state is far larger than that cache (`roofline_streaming`:
N = 151,000,000 float parameters, float gradients, GA), timed the same way.
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
STREAMING_LEG = dict(N=151_000_000, W=8, n_bufs=8, steps=300, warmup=24)   # Transformer-XL-base size (Sec. 6)
ALU_PEAK_TLOPS = 78.65         # fp32 vector 157.3 TFLOP/s / 2 flop per lane-operation
# VALU lane-operations per parameter-update of the persistent kernel (SQ_INSTS_VALU * 64 / updates, profiles/)
VALU_PER_UPDATE = {"ga": 106.7, "ga_hinge": 106.7}
# Bytes per fused-update launch between the L2 and the fabric, measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE
# scaled by a copy of known size; profiles/apply_kernel_cfg3.md).  The counters sit in front of the memory-side
# cache, so hits in that cache are included.  Valid for the kernel source with this hash only.
TRAFFIC = {
    ("cfg3", "ga", 25_557_032): {"bytes": 920040674, "read": 511127518, "written": 408913156, "kernels_sha256": "3f185de6b5c57bdf"},
    ("cfg3", "ga", 151_000_000): {"bytes": 5435414330, "read": 3019394769, "written": 2416019561, "kernels_sha256": "3f185de6b5c57bdf"},
}
BYTES_PER_UPDATE = {           # algorithmic bytes per parameter per arrival, fused update
    ("ga", "f32"): 36, ("ga", "bf16"): 34, ("ga_hinge", "f32"): 36, ("ga_hinge", "bf16"): 34,
    ("asgd", "f32"): 20, ("sa", "f32"): 20, ("sa_step", "f32"): 20,
    ("asgd", "bf16"): 18, ("sa", "bf16"): 18, ("sa_step", "bf16"): 18,
}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=None, help="arrivals to time (default: the workload's own count)")
    p.add_argument("--warmup", type=int, default=None,
                   help="untimed arrivals before the timed ones (default: 100 for the gradient-buffer workloads; one "
                        "pass of the workload's own count for the persistent-kernel workloads, whose first launch of "
                        "a given length runs slower than the following ones)")
    p.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    p.add_argument("--n", type=int, default=None, help="override the workload's number of parameters")
    p.add_argument("--workers", type=int, default=None, help="override the workload's number of workers")
    p.add_argument("--bufs", type=int, default=None, help="buffer workloads: override the number of gradient buffers")
    p.add_argument("--resident-mib", type=float, default=None,
                   help="fused-update workloads: MiB of theta, v, m kept in the memory-side cache (library default 240)")
    p.add_argument("--no-streaming-leg", action="store_true",
                   help="default workload only: skip the second leg at N = 151,000,000")
    p.add_argument("--family", default="momentum", choices=["momentum", "dana", "adam"],
                   help="master algorithm family: Alg. 2-5, Alg. 6-8 or Alg. 9-11")
    p.add_argument("--gap-scope", default="parameter", choices=["parameter", "layer", "global"],
                   help="parameter-wise Gap (Eq. 5), layer-wise (Eq. 4, the workload's tensor table) or global (Def. 1)")
    p.add_argument("--mode", default="ga", choices=["ga", "ga_hinge", "sa", "sa_step", "asgd"])
    p.add_argument("--diag-every", type=int, default=250, help="Gap statistics every this many arrivals (0: never)")
    p.add_argument("--queue", type=int, default=0,
                   help="buffer workloads: apply the arrivals as queues of this many per launch (the persistent kernel "
                        "fed from the gradient buffers) instead of one launch per arrival")
    p.add_argument("--ceiling", action="store_true",
                   help="instead of a workload, measure what the part delivers for the kernels' access pattern and "
                        "instruction mix (stream counts at --n floats per array, default 151,000,000; vector "
                        "instruction rates) and print them as one JSON line")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--calibration-copy", action="store_true",
                   help="after the timed region run three plain device copies of N floats (known size: 4N bytes read, "
                        "4N written) so that a counter profile of this command can be scaled")
    p.add_argument("--cpu-slice", type=int, default=1 << 23, help="parameters in the CPU-oracle sample")
    p.add_argument("--cpu-steps", type=int, default=6000, help="arrivals in the CPU-oracle sample")
    return p.parse_args()


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


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
    by_worker = cfg["pick"] == "worker"
    O.run_buffers(sched[:8], bufs, pick_by_worker=by_worker)       # touch the pages
    n_one = min(128, (n_steps - 8) // 4)                            # a short single-thread leg first
    cores = oracle.num_threads()
    oracle.set_num_threads(1)
    t0 = time.perf_counter()
    O.run_buffers(sched[8:8 + n_one], bufs, pick_by_worker=by_worker)
    dt1 = time.perf_counter() - t0
    oracle.set_num_threads(cores)
    t0 = time.perf_counter()
    O.run_buffers(sched[8 + n_one:], bufs, pick_by_worker=by_worker)
    dt = time.perf_counter() - t0
    n_all = n_steps - 8 - n_one
    return {"value": float(n_slice) * n_all / dt / 1e9, "unit": "G param-updates/s", "cores": cores, "kind": "oracle",
            "value_1_core": float(n_slice) * n_one / dt1 / 1e9, "cpu": cpu_model(),
            "sample": "contiguous slice of %d parameters, all %d workers, the same schedule and gradient recipe: "
                      "%d arrivals on %d threads (%.1f s) after %d arrivals on one thread (%.1f s)"
                      % (n_slice, W, n_all, cores, dt, n_one, dt1)}


def kernels_hash():
    """Hash of the sources of the fused-update kernel (its own file, the shared device header and the header with the
    layout of the state arrays)."""
    import hashlib
    h = hashlib.sha256()
    for name in ("ga_device.h", "ga_apply.hip", "ga_internal.h"):
        h.update(open(os.path.join(ROOT, "paper_1909_10802_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def measured_copy_rate(torch, src):
    """GB/s (bytes read + bytes written) of a plain device copy of the parameter vector: median of 20 timed copies
    after 3 untimed ones.  A reference point for the part's streaming rate, beside the published HBM peak."""
    dst = torch.empty_like(src)
    times = []
    for i in range(23):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dst.copy_(src)
        e1.record()
        e1.synchronize()
        if i >= 3:
            times.append(e0.elapsed_time(e1))
    times.sort()
    return 2.0 * src.numel() * src.element_size() / (times[len(times) // 2] * 1e-3) / 1e9


def bench_fused(args, cfg, torch, ga, ga_inputs):
    """Workloads with precomputed gradient buffers: one fused-update launch per arrival."""
    N, W, seed = cfg["N"], cfg["W"], cfg["seed"]
    dev = "cuda:0"
    K, Wm = args.steps, args.warmup
    bufs = ga_inputs.device_gradient_buffers(cfg["n_bufs"], N, seed, cfg["grad_std"], cfg["grad_dtype"], dev)
    src = ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER if cfg["pick"] == "worker" else ga.GA_PICK_BY_ARRIVAL)
    sched = ga.ga_simulate_schedule(W, K + Wm + 1, ga_inputs.DIST_CODES[cfg["dist"]], cfg["sigma"], seed)
    eta = 0.01 if args.family == "adam" else cfg["eta"]
    scope_kw = {}
    if args.gap_scope == "global":
        scope_kw = dict(gap_scope=ga.GA_GAP_GLOBAL)
    elif args.gap_scope == "layer":
        scope_kw = dict(layer_sizes=ga_inputs.tensor_sizes(N, cfg.get("n_tensors", 161), seed))
    M = ga.Master(N, W, eta=eta, gamma=cfg["gamma"], mode=args.mode, device=dev, family=args.family,
                  track_gap=(args.diag_every > 0), **scope_kw)
    if args.resident_mib is not None:
        ga.ga_set_resident_bytes(M.ctx, int(args.resident_mib * (1 << 20)))
    resident = ga.ga_get_resident_bytes(M.ctx)
    M.run_schedule(sched[:Wm], src)
    if args.diag_every > 0:
        M.diagnostics(int(sched[0]))
    torch.cuda.synchronize()

    seg = args.diag_every if args.diag_every > 0 else K
    events = []
    n_seg = (K + seg - 1) // seg
    reports = torch.zeros((n_seg, ga.DIAG_BYTES), dtype=torch.uint8, device=dev)   # one Gap report per segment
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
        if args.diag_every > 0:                                    # the Gap the next arrival will meet; nothing waits
            M.diagnostics_async(int(sched[Wm + done]), reports[len(events) - 1])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    last_diag = ga.diag_from_device(reports[n_seg - 1]) if args.diag_every > 0 else None

    kernel_ms = sum(a.elapsed_time(b) for a, b in events) / K      # average per launch, on the kernel's stream
    bpu = BYTES_PER_UPDATE[(args.mode, cfg["grad_dtype"])]
    if args.mode in ("asgd", "sa", "sa_step") and args.diag_every > 0:
        bpu += 12                                                   # gap tracking: m read + write, snapshot write
    if args.family != "momentum":
        bpu += 8                                                    # one more state array read and written
    if args.gap_scope != "parameter":
        # inside one run_schedule call the update pass reads the next worker's snapshot instead of this
        # worker's and prepares the next norms: 36 B as for the parameter-wise Gap; only the first arrival
        # of a call needs the separate reduction pass over theta, snapshot and m (12 B)
        bpu += 12.0 * len(events) / K
    achieved = bpu * N / (kernel_ms * 1e-3) / 1e9
    theta = M.theta()
    finite = bool(torch.isfinite(theta).all().item())
    copy_gbs = measured_copy_rate(torch, theta)
    if args.calibration_copy:
        dst = torch.empty(N, dtype=torch.float32, device=dev)
        for _ in range(3):
            dst.copy_(theta)
        torch.cuda.synchronize()
    t = TRAFFIC.get((args.workload, args.mode, N))
    traffic = t["bytes"] if t and t["kernels_sha256"] == kernels_hash() and args.gap_scope == "parameter" else None
    # of the algorithmic bytes, the part that HBM itself has to serve: the kernel keeps a leading part of theta, v, m
    # (ga_get_resident_bytes in all; each kept float saves one read and one write per arrival) in the memory-side cache
    n_hot = {"momentum": 3 if (args.mode in ("ga", "ga_hinge") or args.diag_every > 0) else 2}.get(args.family, 2)
    kept = min(resident, 4 * N * n_hot)
    hbm_only_bpu = bpu - 2.0 * kept / N
    roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic if args.family == "momentum" else None,
            "hbm_only_bytes_per_update": hbm_only_bpu, "hbm_only_GBs": hbm_only_bpu * N / (kernel_ms * 1e-3) / 1e9,
            "hbm_only_frac": hbm_only_bpu * N / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "cache_resident_bytes": kept,
            "kernel": ("layer_gap_kernel + layer_apply_kernel (+ layer_partial_kernel on the first arrival of a call)" if args.gap_scope != "parameter"
                       else "apply_kernel" if args.family == "momentum" else "family_apply_kernel"), "bytes_per_update": bpu, "avg_launch_ms": kernel_ms,
            "algorithmic_bytes_per_launch": int(round(bpu * N)),
            "copy_GBs": copy_gbs, "frac_of_copy": achieved / copy_gbs}
    desc = ("%s: N=%d float parameters, %d workers, %s iteration times, %d %s gradient buffers picked by %s, one "
            "fused-update launch per arrival, family %s, mode %s" % (args.workload, N, W, cfg["dist"], cfg["n_bufs"],
                                                                     cfg["grad_dtype"], cfg["pick"], args.family,
                                                                     args.mode))
    extra = {"hbm_pct_of_peak": 100.0 * achieved / HBM_PEAK_GBS, "theta_finite": finite,
             "mean_gap_last": None if last_diag is None else last_diag["mean_graw"] + 1.0}
    M.close()
    del M, bufs, src, theta
    torch.cuda.empty_cache()
    return wall, roof, desc, extra


def streaming_leg(args, cfg, torch, ga, ga_inputs):
    """The fused update where the state is far larger than the memory-side cache: the same kernel, gradient recipe
    and timing as the main leg at N = 151,000,000 (float gradients, a few workers so that it allocates fast)."""
    leg = dict(STREAMING_LEG)
    c2 = dict(cfg, N=leg["N"], W=leg["W"], n_bufs=leg["n_bufs"])
    a2 = argparse.Namespace(**vars(args))
    a2.steps, a2.warmup, a2.diag_every, a2.calibration_copy = leg["steps"], leg["warmup"], 0, False
    wall, roof, desc, _ = bench_fused(a2, c2, torch, ga, ga_inputs)
    keys = ("achieved", "peak", "unit", "frac", "traffic", "kernel", "bytes_per_update", "avg_launch_ms",
            "algorithmic_bytes_per_launch", "hbm_only_bytes_per_update", "hbm_only_GBs", "hbm_only_frac",
            "cache_resident_bytes", "copy_GBs", "frac_of_copy")
    out = {"N": leg["N"], "n_workers": leg["W"], "steps": leg["steps"], "warmup": leg["warmup"], "workload": desc,
           "G_param_updates_per_s": leg["N"] * leg["steps"] / wall / 1e9}
    out.update({k: roof[k] for k in keys})
    return out


def bench_queue(args, cfg, torch, ga, ga_inputs):
    """Buffer workloads with the arrivals applied as queues of --queue per launch (results identical to one
    launch per arrival; theta, v, m are read and written once per queue instead of once per arrival)."""
    N, W, seed = cfg["N"], cfg["W"], cfg["seed"]
    dev = "cuda:0"
    K, Wm, Q = args.steps, args.warmup, args.queue
    bufs = ga_inputs.device_gradient_buffers(cfg["n_bufs"], N, seed, cfg["grad_std"], cfg["grad_dtype"], dev)
    src = ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER if cfg["pick"] == "worker" else ga.GA_PICK_BY_ARRIVAL,
                           persistent=True)
    sched = ga.ga_simulate_schedule(W, K + Wm + 1, ga_inputs.DIST_CODES[cfg["dist"]], cfg["sigma"], seed)
    eta = 0.01 if args.family == "adam" else cfg["eta"]
    track = args.mode in ("ga", "ga_hinge")
    M = ga.Master(N, W, eta=eta, gamma=cfg["gamma"], mode=args.mode, device=dev, family=args.family)
    M.run_schedule(sched[:Wm], src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    n_launch = 0
    for done in range(0, K, Q):
        M.run_schedule(sched[Wm + done:Wm + min(done + Q, K)], src)
        n_launch += 1
    e1.record()
    last_diag = M.diagnostics(int(sched[Wm + K])) if track else None
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_s = e0.elapsed_time(e1) * 1e-3
    g_bytes = 4 if cfg["grad_dtype"] == "f32" else 2
    per_arrival = g_bytes + (8 if track else 0) + (8 if args.family == "dana" else 0)
    per_launch = 4 * 2 * ((3 if track else 2) + (1 if args.family == "adam" else 0))
    bpu = per_arrival + per_launch * n_launch / K
    ach = bpu * N * K / kernel_s / 1e9
    roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "traffic": None, "kernel": "persistent_kernel (gradient buffers)", "bytes_per_update": bpu,
            "avg_launch_ms": kernel_s * 1e3 / n_launch, "arrivals_per_launch": Q,
            "algorithmic_bytes_per_launch": int(round(bpu * N * K / n_launch))}
    desc = ("%s: N=%d float parameters, %d workers, %s iteration times, %d %s gradient buffers picked by %s, queues of "
            "%d arrivals per launch, family %s, mode %s" % (args.workload, N, W, cfg["dist"], cfg["n_bufs"],
                                                            cfg["grad_dtype"], cfg["pick"], Q, args.family, args.mode))
    theta = M.theta()
    if args.calibration_copy:
        dst = torch.empty(N, dtype=torch.float32, device=dev)
        for _ in range(3):
            dst.copy_(theta)
        torch.cuda.synchronize()
    extra = {"theta_finite": bool(torch.isfinite(theta).all().item()),
             "mean_gap_last": None if last_diag is None else last_diag["mean_graw"] + 1.0}
    return wall, roof, desc, extra


def bench_persistent(args, cfg, torch, ga, ga_inputs):
    """Workloads with the in-kernel quadratic-plus-noise source: the persistent multi-arrival kernel."""
    N, W, seed = cfg["N"], cfg["W"], cfg["seed"]
    dev = "cuda:0"
    K, Wm = args.steps, args.warmup
    a, ts = ga_inputs.device_curvatures(N, seed, dev), ga_inputs.device_optimum(N, seed, dev)
    src = ga.quadratic_source(a, ts, seed, 0.01, persistent=True)
    sched = ga.ga_simulate_schedule(W, K + Wm + 1, ga_inputs.DIST_CODES[cfg["dist"]], cfg["sigma"], seed)
    eta = 0.01 if args.family == "adam" else cfg["eta"]
    M = ga.Master(N, W, eta=eta, gamma=cfg["gamma"], mode=args.mode, device=dev, family=args.family)
    M.run_schedule(sched[:Wm], src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    M.run_schedule(sched[Wm:Wm + K], src)
    e1.record()
    last_diag = M.diagnostics(int(sched[Wm + K])) if args.mode in ("ga", "ga_hinge") else None
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_s = e0.elapsed_time(e1) * 1e-3                            # all chunks of the schedule
    ups = N * K / kernel_s
    if args.mode in VALU_PER_UPDATE and args.family == "momentum":
        ach = ups * VALU_PER_UPDATE[args.mode] / 1e12
        roof = {"bound": "alu", "achieved": ach, "peak": ALU_PEAK_TLOPS, "unit": "T lane-op/s",
                "frac": ach / ALU_PEAK_TLOPS, "traffic": None, "kernel": "persistent_kernel",
                "valu_ops_per_update": VALU_PER_UPDATE[args.mode], "hbm_GBs_at_8B_per_update": 8 * ups / 1e9}
    else:
        bpu = 16 if args.family == "dana" else 8       # snapshot row (and DANA's worker momentum row) read + written
        ach = bpu * ups / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": None, "kernel": "persistent_kernel", "bytes_per_update": bpu}
    roof["kernel_ms_total"] = kernel_s * 1e3
    theta = M.theta()
    desc = ("%s: N=%d float parameters, %d workers, %s iteration times, quadratic-plus-noise gradients generated in "
            "the persistent multi-arrival kernel, family %s, mode %s" % (args.workload, N, W, cfg["dist"], args.family,
                                                                        args.mode))
    extra = {"theta_finite": bool(torch.isfinite(theta).all().item()),
             "mean_gap_last": None if last_diag is None else last_diag["mean_graw"] + 1.0}
    return wall, roof, desc, extra


def cpu_baseline_quadratic(cfg, mode, n_slice, n_steps):
    """Oracle on a contiguous slice of a quadratic-source workload (it generates the noise itself)."""
    import ga_inputs
    import oracle
    W, seed = cfg["W"], cfg["seed"]
    n_slice = min(n_slice, cfg["N"], 1 << 20)
    n_steps = min(n_steps, cfg["T"], 400)
    a, ts = ga_inputs.curvatures(n_slice, seed), ga_inputs.optimum(n_slice, seed)
    sched = oracle.simulate_schedule(W, n_steps, ga_inputs.DIST_CODES[cfg["dist"]], cfg["sigma"], seed)
    modes = dict(ga=oracle.MODE_GA, ga_hinge=oracle.MODE_GA_HINGE, sa=oracle.MODE_SA, sa_step=oracle.MODE_SA_STEP,
                 asgd=oracle.MODE_ASGD)
    O = oracle.Master(n_slice, W, modes[mode], oracle.Hyper(cfg["eta"], cfg["gamma"]))
    O.run_quadratic(sched[:8], a, ts, seed)
    t0 = time.perf_counter()
    O.run_quadratic(sched[8:], a, ts, seed)
    dt = time.perf_counter() - t0
    return {"value": float(n_slice) * (n_steps - 8) / dt / 1e9, "unit": "G param-updates/s",
            "cores": oracle.num_threads(), "kind": "oracle", "cpu": cpu_model(),
            "sample": "first %d parameters, all %d workers, %d arrivals of the same schedule (%.1f s)"
                      % (n_slice, W, n_steps - 8, dt)}


def ceiling(args, torch, ga):
    """Rates of the measurement aids of the library (ga_probe_streams, ga_probe_valu), events on the current stream."""
    dev = "cuda:0"
    n = (args.n or 151_000_000) // 4 * 4
    bufs = [torch.full((n,), 0.5 + i, dtype=torch.float32, device=dev) for i in range(9)]

    def timed(launch, reps):
        for _ in range(3):
            launch()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            launch()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    streams = {}
    for r, w in ((1, 0), (5, 0), (0, 1), (0, 4), (1, 1), (2, 2), (4, 4), (5, 1), (5, 2), (5, 4)):
        s = timed(lambda: ga.ga_probe_streams(bufs[:r], bufs[5:5 + w], n), 20)
        streams["%dr%dw" % (r, w)] = 4.0 * (r + w) * n / s / 1e9
    # the update's own pattern: four arrays rewritten in place and one more read; then the same with the first three
    # laid out as the library lays out theta, v, m (interleaved by tiles of 8192 floats in one buffer)
    s = timed(lambda: ga.ga_probe_streams(bufs[:5], bufs[:4], n), 20)
    streams["5r4w_in_place"] = 4.0 * 9 * n / s / 1e9
    tile = 8192
    state = torch.full((3 * ((n + tile - 1) // tile) * tile,), 0.5, dtype=torch.float32, device=dev)
    tiled = [state, state[tile:], state[2 * tile:], bufs[3], bufs[4]]
    s = timed(lambda: ga.ga_probe_streams(tiled, tiled[:4], n, tiled=True), 20)
    streams["5r4w_in_place_state_tiled"] = 4.0 * 9 * n / s / 1e9
    del bufs, state, tiled
    torch.cuda.empty_cache()
    # Data held in the memory-side cache: two arrays of the cfg3 size (204 MB together) accessed without the hint,
    # alone and inside the fused update's mix: theta, v, m, snapshot updated in place, the gradient read, with the
    # snapshot and the gradient taken from a pool in turn as the arrivals of different workers do.
    nr = 25_557_032
    fixed = [torch.full((nr,), 0.5 + i, dtype=torch.float32, device=dev) for i in range(3)]        # theta, v, m
    pool = [torch.full((nr,), 3.5 + i, dtype=torch.float32, device=dev) for i in range(16)]        # snapshots, gradients
    turn = [0]

    def mix(n_resident):
        i = turn[0] = (turn[0] + 2) % len(pool)
        arrays = fixed + [pool[i], pool[i + 1]]
        ga.ga_probe_streams(arrays, arrays[:4], nr, n_resident=n_resident)

    resident = {}
    for name, r, w in (("2r0w", 2, 0), ("2r2w_in_place", 2, 2)):
        s = timed(lambda: ga.ga_probe_streams(fixed[:r], fixed[:w], nr, n_resident=2), 40)
        resident[name] = 4.0 * (r + w) * nr / s / 1e9
    resident["5r4w_in_place"] = 4.0 * 9 * nr / timed(lambda: mix(2), 48) / 1e9
    resident["5r4w_in_place_all_streamed"] = 4.0 * 9 * nr / timed(lambda: mix(0), 48) / 1e9
    del fixed, pool
    torch.cuda.empty_cache()
    out = torch.zeros(1, dtype=torch.int32, device=dev)
    blocks, iters = 8 * torch.cuda.get_device_properties(0).multi_processor_count, 4096
    valu = {}
    for op in ga.PROBE_OPS:
        s = timed(lambda: ga.ga_probe_valu(op, blocks, iters, out), 5)
        valu[op] = blocks * 256.0 * iters * 8 / s / 1e12
    return {"n_floats_per_array": n, "stream_GBs": streams,
            "resident_stream_GBs": dict(resident, n_floats_per_array=nr, note="the first two arrays are accessed without the non-temporal hint"),
            "valu_T_lane_ops_per_s": valu,
            "valu_probe": "%d blocks of 256 threads x %d iterations x 8 independent instructions" % (blocks, iters),
            "hbm_peak_GBs": HBM_PEAK_GBS, "alu_peak_T_lane_ops_per_s": ALU_PEAK_TLOPS}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on one GPU only (the master update would shard by parameter range with "
              "no exchange between shards, but that is not implemented). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import ga_inputs
    import paper_1909_10802_amd as ga

    if args.ceiling:
        torch.cuda.set_device(0)
        print(json.dumps({"ceiling": ceiling(args, torch, ga)}))
        return
    cfg = dict(ga_inputs.WORKLOADS[args.workload])
    if args.n is not None:
        cfg["N"] = args.n
    if args.workers is not None:
        cfg["W"] = args.workers
    if args.bufs is not None:
        if cfg["source"] != "buffers":
            sys.exit("bench.py: --bufs is for the gradient-buffer workloads")
        cfg["n_bufs"] = args.bufs
    if args.steps is None:
        args.steps = cfg["T"]
    if args.warmup is None:
        args.warmup = 100 if cfg["source"] == "buffers" else cfg["T"]
    torch.cuda.set_device(0)
    fused = cfg["source"] == "buffers"
    if not fused and args.gap_scope != "parameter":
        sys.exit("bench.py: the persistent-kernel workloads use the parameter-wise Gap")
    if args.queue and (not fused or args.gap_scope != "parameter"):
        sys.exit("bench.py: --queue is for the gradient-buffer workloads with the parameter-wise Gap")
    run = bench_queue if (fused and args.queue) else bench_fused if fused else bench_persistent
    wall, roof, desc, extra = run(args, cfg, torch, ga, ga_inputs)
    N, K = cfg["N"], args.steps
    out = {
        "metric": "G param-updates/s and achieved HBM GB/s (% of peak), GA fused update",
        "value": N * K / wall / 1e9,
        "unit": "G param-updates/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": desc, "N": N, "n_workers": cfg["W"], "family": args.family, "mode": args.mode, "gap_scope": args.gap_scope,
                   "grad_dtype": cfg["grad_dtype"], "eta": cfg["eta"], "gamma": cfg["gamma"],
                   "diag_every": args.diag_every if fused else None, "seed": cfg["seed"]},
        "roofline": roof,
    }
    out.update(extra)
    default_leg = (run is bench_fused and args.workload == "cfg3" and args.family == "momentum" and args.mode == "ga"
                   and args.gap_scope == "parameter" and args.n is None)
    if default_leg and not args.no_streaming_leg:
        out["roofline_streaming"] = streaming_leg(args, cfg, torch, ga, ga_inputs)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = (cpu_baseline if fused else cpu_baseline_quadratic)(cfg, args.mode, args.cpu_slice,
                                                                                  args.cpu_steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
