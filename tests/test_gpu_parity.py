"""GPU-vs-oracle parity of the master update, through the C ABI (needs an MI355X).

Small and medium sizes: every element of theta, v, m and all snapshots is
compared after single teacher-forced steps (relative 1e-6) and after whole
trajectories (relative L2 of theta <= 1e-5; integer bookkeeping bit exact).
"""
import numpy as np
import pytest
import torch

import ga_inputs
import oracle
import paper_1909_10802_amd as ga
from gpu_util import (DEV, MODE_NAMES, MODES, RTOL_TRAJ_L2, assert_step_close, bits_equal, compare_masters, dev,
                      gpu_state, host, load_state, rel_l2)

pytestmark = pytest.mark.gpu

SIZES = [1, 3, 4, 5, 255, 1024, 2048 + 5, 100_003]


# ------------------------------------------------------------------ noise generator
@pytest.mark.parametrize("seed,k,j0,n", [(1, 1, 0, 1 << 20), (2**40 + 3, 2**33 + 5, 2**34 + 1, 100_001), (7, 9, 3, 5)])
def test_noise_bit_exact(seed, k, j0, n):
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    ga.ga_noise_fill(seed, k, j0, n, out)
    assert bits_equal(host(out), oracle.noise_f32(seed, k, j0, n)) == 0


def test_noise_transform_exhaustive():
    # every radius input (the 2^23 values of xa >> 9) and every angle input (the 2^25 values of xb >> 7)
    def run(xa, xb):
        zc, zs = torch.empty(xa.size, dtype=torch.float32, device=DEV), torch.empty(xa.size, dtype=torch.float32, device=DEV)
        ga.ga_box_muller_raw(dev(xa.view(np.int32)), dev(xb.view(np.int32)), zc, zs)
        rc, rs = oracle.box_muller_raw(xa, xb)
        assert bits_equal(host(zc), rc) == 0 and bits_equal(host(zs), rs) == 0
    m = np.arange(1 << 23, dtype=np.uint32)
    for xb in (0x00000000, 0x5A5A5A5A, 0xFFFFFFFF):
        run(m << np.uint32(9), np.full(m.size, xb, np.uint32))
    for lo in range(0, 1 << 25, 1 << 23):
        f = np.arange(lo, lo + (1 << 23), dtype=np.uint32)
        run(np.full(f.size, 0x9E3779B9, np.uint32), f << np.uint32(7))


# ------------------------------------------------------------------ single step, teacher forced
@pytest.mark.parametrize("mode", MODES, ids=[MODE_NAMES[m] for m in MODES])
@pytest.mark.parametrize("N", SIZES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_step(mode, N, dtype):
    W, k, tau = 3, 57, 5
    theta, v, m, snaps = ga_inputs.random_state(N, W, seed=N)
    g32 = (0.3 * ga_inputs.rng(N, 7).standard_normal(N)).astype(np.float32)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(g32)
        g_ref = oracle.bf16_to_f32(bits)
        g_dev = dev(bits.view(np.int16)).view(torch.bfloat16)
    else:
        g_ref, g_dev = g32, dev(g32)
    it = np.array([k - 1, k - tau, 3], dtype=np.uint64)       # worker 1 arrives with delay tau
    M = ga.Master(N, W, mode=mode, track_gap=True)
    load_state(M, theta, v, m, snaps, k - 1, it)
    M.apply(1, g_dev)
    O = oracle.Master(N, W, mode, oracle.Hyper(), track_gap=True)
    O.theta[:], O.v[:], O.m[:], O.snaps[:], O.k, O.iter[:] = theta, v, m, snaps, k - 1, it
    assert O.apply(1, g_ref) == tau
    compare_masters(M, O, "N=%d %s %s" % (N, MODE_NAMES[mode], dtype))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("offset", [1, 2, 3])
def test_single_step_misaligned_gradient(dtype, offset):
    N, W = 10_007, 2
    theta, v, m, snaps = ga_inputs.random_state(N, W, seed=4)
    g32 = ga_inputs.rng(4, 7).standard_normal(N + 8).astype(np.float32)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(g32)
        g_ref = oracle.bf16_to_f32(bits)[offset:offset + N]
        g_dev = dev(bits.view(np.int16)).view(torch.bfloat16)[offset:offset + N]
    else:
        g_ref, g_dev = g32[offset:offset + N], dev(g32)[offset:offset + N]
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    load_state(M, theta, v, m, snaps, 10, np.array([4, 10], np.uint64))
    M.apply(0, g_dev)
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
    O.theta[:], O.v[:], O.m[:], O.snaps[:], O.k, O.iter[:] = theta, v, m, snaps, 10, [4, 10]
    O.apply(0, np.ascontiguousarray(g_ref))
    compare_masters(M, O, "misaligned %s +%d" % (dtype, offset))


def test_first_arrival_and_special_values():
    # k = 1 (m-hat taken as 0), then denormal / huge / zero / non-finite inputs in every array
    N, W = 4096 + 3, 2
    rng = np.random.default_rng(0)
    specials = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-39, 1e-38, 1.17549435e-38, 3e38, -3e38, 1e-20, 1e20,
                         np.inf, -np.inf, np.nan], dtype=np.float32)
    for mode in (ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE, ga.GA_MODE_SA):
        M = ga.Master(N, W, mode=mode, track_gap=True)
        O = oracle.Master(N, W, mode, oracle.Hyper(), track_gap=True)
        g = rng.standard_normal(N).astype(np.float32)
        M.apply(0, dev(g))
        O.apply(0, g)
        compare_masters(M, O, "first arrival")
        theta, v, m, snaps = ga_inputs.random_state(N, W, seed=2)
        for arr in (theta, v, snaps[0], snaps[1]):
            arr[rng.integers(0, N, 400)] = rng.choice(specials, 400)
        m[rng.integers(0, N, 400)] = np.abs(rng.choice(specials, 400))
        g[rng.integers(0, N, 400)] = rng.choice(specials, 400)
        load_state(M, theta, v, m, snaps, 1, np.array([1, 0], np.uint64))
        O.theta[:], O.v[:], O.m[:], O.snaps[:] = theta, v, m, snaps
        M.apply(1, dev(g))
        O.apply(1, g)
        compare_masters(M, O, "special values " + MODE_NAMES[mode], exact=False)
        th = gpu_state(M)[0]
        assert bits_equal(np.nan_to_num(th, nan=7.0), np.nan_to_num(O.theta, nan=7.0)) == 0


# ------------------------------------------------------------------ trajectories
@pytest.mark.parametrize("mode", MODES, ids=[MODE_NAMES[m] for m in MODES])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_trajectory_buffers(mode, dtype):
    N, W, T, n_bufs = 20_011, 6, 150, 4
    bufs = ga_inputs.gradient_buffers(n_bufs, N, seed=11, std=0.3)
    sched = ga.ga_simulate_schedule(W, T, seed=11)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(bufs).reshape(n_bufs, N)
        ref_bufs = oracle.bf16_to_f32(bits).reshape(n_bufs, N)
        dbufs = [dev(b.view(np.int16)).view(torch.bfloat16) for b in bits]
    else:
        ref_bufs, dbufs = bufs, [dev(b) for b in bufs]
    for pick in (ga.GA_PICK_BY_WORKER, ga.GA_PICK_BY_ARRIVAL):
        M = ga.Master(N, W, mode=mode, track_gap=True)
        M.run_schedule(sched, ga.buffer_source(dbufs, pick))
        O = oracle.Master(N, W, mode, oracle.Hyper(), track_gap=True)
        O.run_buffers(sched, np.ascontiguousarray(ref_bufs), pick_by_worker=(pick == ga.GA_PICK_BY_WORKER))
        compare_masters(M, O, "buffers %s %s" % (MODE_NAMES[mode], dtype))
        assert rel_l2(host(M.theta()), O.theta) <= RTOL_TRAJ_L2


@pytest.mark.parametrize("mode", MODES, ids=[MODE_NAMES[m] for m in MODES])
@pytest.mark.parametrize("persistent", [True, False], ids=["persistent", "per_arrival"])
def test_trajectory_quadratic(mode, persistent):
    N, W, T, seed = 30_002, 8, 200, 5          # N % 4 == 2: ragged tail
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    M = ga.Master(N, W, mode=mode)
    scratch = torch.empty(N, dtype=torch.float32, device=DEV)
    src = ga.quadratic_source(dev(a), dev(ts), seed, 0.01, persistent, scratch)
    M.run_schedule(sched[:77], src)            # two calls: the step counter carries over
    M.run_schedule(sched[77:], src)
    O = oracle.Master(N, W, mode, oracle.Hyper())
    O.run_quadratic(sched, a, ts, seed)
    keep_m = mode in (ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE)
    compare_masters(M, O, "quadratic %s" % MODE_NAMES[mode], keep_m=keep_m)
    assert rel_l2(host(M.theta()), O.theta) <= RTOL_TRAJ_L2


def test_persistent_repeated_worker_and_chunk_boundary():
    # the same worker several times in a row (its snapshot is forwarded in registers) and
    # a schedule longer than one table chunk (8192 arrivals per launch)
    N, W, seed = 1000 + 1, 3, 9
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    rng = np.random.default_rng(1)
    sched = np.concatenate([[0, 0, 0, 1, 1, 0, 2, 2, 2, 2, 0],
                            np.repeat(rng.integers(0, W, 4200), 2)]).astype(np.uint32)[:8192 + 37]
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    M.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed))
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
    O.run_quadratic(sched, a, ts, seed)
    compare_masters(M, O, "repeats + chunks")


def test_quadratic_gradient_entry_point():
    N, W, seed = 12_345, 4, 3
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    src = ga.quadratic_source(dev(a), dev(ts), seed, 0.01)
    M.run_schedule(np.array([0, 1, 2, 1], np.uint32), src)
    g = torch.empty(N, dtype=torch.float32, device=DEV)
    ga.ga_quadratic_gradient(M.ctx, 2, src, g)
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
    O.run_quadratic(np.array([0, 1, 2, 1], np.uint32), a, ts, seed)
    ref = oracle.quadratic_gradient(O.snaps[2], a, ts, seed, k=5)
    assert bits_equal(host(g), ref) == 0
    assert M.k == 4                                            # state untouched


def test_single_worker_modes_coincide():
    # no master update between send and receive: every penalty is exactly 1
    N, T, seed = 5000, 40, 2
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    outs = []
    for mode in MODES:
        M = ga.Master(N, 1, mode=mode)
        M.run_schedule(np.zeros(T, np.uint32), ga.quadratic_source(dev(a), dev(ts), seed))
        outs.append(host(M.theta()))
    for o in outs[1:]:
        assert bits_equal(o, outs[0]) == 0


# ------------------------------------------------------------------ diagnostics
@pytest.mark.parametrize("N", [1, 7, 4096, 1_000_003])
def test_diagnostics(N):
    W, seed = 4, 21
    theta, v, m, snaps = ga_inputs.random_state(N, W, seed)
    if N > 100:
        snaps[2, 5] = np.inf
        theta[9] = np.nan
        snaps[2, 11:20] = theta[11:20]                          # zero gap
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    it = np.array([100, 90, 50, 1], np.uint64)
    load_state(M, theta, v, m, snaps, 100, it)
    for w in (0, 2):
        d = M.diagnostics(w)
        r = oracle.gap_statistics(theta, m, snaps[w], 100, oracle.Hyper())
        assert d["n_nonfinite"] == r["n_nonfinite"]
        assert round(d["frac_gt1"] * N) == r["n_gt1"] and round(d["frac_gt0"] * N) == r["n_gt0"]
        assert abs(d["mean_graw"] - r["mean_graw"]) <= 1e-6 * abs(r["mean_graw"])
    # before any arrival: C = eta_max * eps, every gap is zero
    M0 = ga.Master(N, W, mode=ga.GA_MODE_GA)
    d0 = M0.diagnostics(1)
    assert d0 == dict(mean_graw=0.0, frac_gt1=0.0, frac_gt0=0.0, n_nonfinite=0)


def test_diagnostics_counts_are_strict_at_graw_equal_one():
    # beta = 1/2, k = 1: m-hat = 2 m = 1/16, root 1/4; eps = 2^-10, eta_max = 1/2 -> C = 1/8 + 2^-11 exactly.
    # Distances {0, C/2, C, 2C, inf, nan}: Graw = 1 exactly is penalised by the paper's form and not by the hinge form.
    Cc = np.float32(0.125 + 2.0 ** -11)
    diff = np.array([0.0, Cc / 2, -Cc, 2 * Cc, np.inf, np.nan, 0.0], np.float32)
    snap = np.zeros(7, np.float32)
    theta, m, v = diff.copy(), np.full(7, 0.03125, np.float32), np.zeros(7, np.float32)
    M = ga.Master(7, 1, eta=0.5, mode=ga.GA_MODE_GA, beta=0.5, eps=2.0 ** -10)
    load_state(M, theta, v, m, snap[None, :], 1, np.array([1], np.uint64))
    d = M.diagnostics(0)
    r = oracle.gap_statistics(theta, m, snap, 1, oracle.Hyper(eta=0.5, beta=0.5, eps=2.0 ** -10))
    assert (round(d["frac_gt0"] * 7), round(d["frac_gt1"] * 7), d["n_nonfinite"]) == (3, 1, 2)
    assert (r["n_gt0"], r["n_gt1"], r["n_nonfinite"]) == (3, 1, 2)
    assert d["mean_graw"] == r["mean_graw"] == 3.5 / 7


def test_diagnostics_under_sa_with_tracking():
    N, W, T, seed = 50_000, 8, 120, 6
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    M = ga.Master(N, W, mode=ga.GA_MODE_SA, track_gap=True)
    M.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed))
    O = oracle.Master(N, W, oracle.MODE_SA, oracle.Hyper(), track_gap=True)
    O.run_quadratic(sched, a, ts, seed)
    compare_masters(M, O, "SA tracked")
    for w in range(W):
        d, r = M.diagnostics(w), O.gap_statistics(w)
        assert abs(d["mean_graw"] - r["mean_graw"]) <= 1e-6 * abs(r["mean_graw"]) + 1e-300
        assert round(d["frac_gt1"] * N) == r["n_gt1"]


@pytest.mark.parametrize("N", [3, 4097, 2_500_001])
def test_diagnostics_async_writes_the_report_on_the_device(N):
    """ga_diagnostics_async: same statistics as the oracle (App. C.8), written to device memory with no wait; it
    must not disturb the arrivals enqueued around it."""
    W, seed = 3, 33
    theta, v, m, snaps = ga_inputs.random_state(N, W, seed)
    if N > 100:
        snaps[1, 17] = np.inf
        snaps[1, 40:50] = theta[40:50]
    k = 60
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    load_state(M, theta, v, m, snaps, k, np.array([60, 31, 2], np.uint64))
    outs = [M.diagnostics_async(w) for w in (1, 2)]             # two reports in flight, none waited for
    g = ga_inputs.gradient_buffers(1, N, seed)[0]
    M.apply(0, dev(g))                                           # an arrival behind them on the same stream
    for w, out in zip((1, 2), outs):
        d = ga.diag_from_device(out)
        r = oracle.gap_statistics(theta, m, snaps[w], k, oracle.Hyper())
        assert d["n_nonfinite"] == r["n_nonfinite"]
        assert round(d["frac_gt1"] * N) == r["n_gt1"] and round(d["frac_gt0"] * N) == r["n_gt0"]
        assert abs(d["mean_graw"] - r["mean_graw"]) <= 1e-6 * abs(r["mean_graw"])
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
    O.theta, O.v, O.m, O.snaps = theta.copy(), v.copy(), m.copy(), snaps.copy()
    O.k, O.iter = k, np.array([60, 31, 2], np.uint64)
    O.apply(0, g)
    th, vv, mm, sn = gpu_state(M)
    assert_step_close(th, O.theta, "theta after the arrival behind the reports")
    assert_step_close(sn, O.snaps, "snapshots after the arrival behind the reports")
    with pytest.raises(ga.GaError):
        ga.Master(N, W, mode=ga.GA_MODE_SA).diagnostics_async(0)   # m is not maintained


# ------------------------------------------------------------------ state handling
def test_checkpoint_resume_is_bit_identical():
    N, W, T, seed = 40_000, 5, 160, 8
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    src = ga.quadratic_source(dev(a), dev(ts), seed)
    A = ga.Master(N, W, mode=ga.GA_MODE_GA)
    A.run_schedule(sched, src)
    B = ga.Master(N, W, mode=ga.GA_MODE_GA)
    B.run_schedule(sched[:70], src)
    th, v, m, sn = gpu_state(B)
    k, it = B.k, B.iter()
    C2 = ga.Master(N, W, mode=ga.GA_MODE_GA)
    load_state(C2, th, v, m, sn, k, it)
    C2.run_schedule(sched[70:], src)
    for x, y in zip(gpu_state(A), gpu_state(C2)):
        assert bits_equal(x, y) == 0
    assert C2.k == A.k and np.array_equal(C2.iter(), A.iter())


def test_delay_log_keeps_the_most_recent_arrivals():
    # the host keeps the delays of the last 2^20 arrivals only (Sec. 6 runs have 10^5 - 10^6 master steps)
    N, W, kept = 4, 3, 1 << 20
    T = kept + 5000
    a, ts = ga_inputs.curvatures(N, 2), ga_inputs.optimum(N, 2)
    sched = ga.ga_simulate_schedule(W, T, seed=2)
    M = ga.Master(N, W, mode=ga.GA_MODE_SA)
    M.run_schedule(sched[:1000], ga.quadratic_source(dev(a), dev(ts), 2))
    assert np.array_equal(M.delays(), oracle.delays(W, sched[:1000])[0])
    M.run_schedule(sched[1000:], ga.quadratic_source(dev(a), dev(ts), 2))
    torch.cuda.synchronize()
    taus, it = oracle.delays(W, sched)
    got = M.delays()
    assert got.size == kept and np.array_equal(got, taus[-kept:])
    assert M.k == T and np.array_equal(M.iter(), it)
    few = np.empty(7, np.uint64)                                   # fewer than kept: the most recent ones
    n = ga.C.c_uint64()
    assert ga.lib().ga_get_delays(M.ctx, few.ctypes.data_as(ga.C.c_void_p), 7, ga.C.byref(n)) == ga.GA_OK
    assert n.value == kept and np.array_equal(few, taus[-7:])


def test_get_config_returns_what_the_context_runs_with():
    M = ga.Master(1000, 5, eta=0.05, gamma=-0.3, mode=ga.GA_MODE_GA_HINGE, beta=0.99, eps=1e-6, eta_max=0.2, nesterov=True)
    ga.ga_set_lr(M.ctx, 0.0125)
    cfg, eta_k = ga.ga_get_config(M.ctx)
    f = np.float32
    assert (cfg.N, cfg.n_workers, cfg.family, cfg.mode, cfg.nesterov) == (1000, 5, ga.GA_FAMILY_MOMENTUM, ga.GA_MODE_GA_HINGE, 1)
    assert (f(cfg.eta), f(cfg.gamma), f(cfg.beta), f(cfg.eps), f(eta_k)) == (f(0.2), f(-0.3), f(0.99), f(1e-6), f(0.0125))
    A = ga.Master(64, 2, eta=0.01, family=ga.GA_FAMILY_ADAM, adam_beta1=0.8, adam_beta2=0.95, adam_eps=1e-5, track_gap=True)
    cfg, _ = ga.ga_get_config(A.ctx)
    assert (cfg.family, cfg.track_gap, f(cfg.adam_beta1), f(cfg.adam_beta2), f(cfg.adam_eps)) == (ga.GA_FAMILY_ADAM, 1, f(0.8), f(0.95), f(1e-5))


@pytest.mark.parametrize("mode", [ga.GA_MODE_GA, ga.GA_MODE_ASGD], ids=["ga", "asgd"])
def test_resident_budget_changes_no_result(mode):
    # the budget only moves the block thresholds between the four hint paths of the fused update (and of the
    # Gap statistics): every split of a 1 M parameter vector gives the oracle's bits
    N, W, T, seed = 1_000_003, 3, 9, 44
    bufs = ga_inputs.gradient_buffers(2, N, seed, 0.3)
    dbufs = [dev(b) for b in bufs]
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    O = oracle.Master(N, W, mode, oracle.Hyper(), track_gap=True)
    O.run_buffers(sched, bufs)
    ref = O.gap_statistics(1)
    for budget in (0, 1 << 20, 5 << 20, 9 << 20, 11 << 20, 240 << 20):    # theta is 4 MB: none | part of theta | ... | all
        M = ga.Master(N, W, mode=mode, track_gap=True)
        ga.ga_set_resident_bytes(M.ctx, budget)
        assert ga.ga_get_resident_bytes(M.ctx) == budget
        M.run_schedule(sched, ga.buffer_source(dbufs))
        compare_masters(M, O, "budget %d" % budget)
        d = M.diagnostics(1)
        assert d["mean_graw"] == pytest.approx(ref["mean_graw"], rel=1e-6) and round(d["frac_gt1"] * N) == ref["n_gt1"]
        M.close()


def test_theta0_and_setters():
    N, W = 3001, 3
    th0 = ga_inputs.optimum(N, 1)
    M = ga.Master(N, W, mode=ga.GA_MODE_GA, theta0=dev(th0), beta=0.99, eps=1e-6, eta_max=0.2)
    for w in range(W):
        assert bits_equal(host(M.snapshot(w)), th0) == 0
    g = ga_inputs.rng(1, 3).standard_normal(N).astype(np.float32)
    ga.ga_set_lr(M.ctx, 0.05)
    M.apply(0, dev(g))
    M.apply(1, dev(g))
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper(eta=0.2, eta_k=0.05, beta=0.99, eps=1e-6), theta0=th0)
    O.apply(0, g)
    O.apply(1, g)
    compare_masters(M, O, "theta0 + setters")
    for fn, args in [(ga.ga_set_beta_eps, (0.9, 1e-8)), (ga.ga_set_eta_max, (0.1,)), (ga.ga_set_track_gap, (True,)),
                     (ga.ga_set_theta, (dev(th0),))]:
        with pytest.raises(ga.GaError) as e:
            fn(M.ctx, *args)
        assert e.value.status == ga.GA_ERR_STATE


def test_errors_leave_state_unchanged():
    N, W = 1000, 2
    M = ga.Master(N, W, mode=ga.GA_MODE_ASGD)
    g = dev(np.ones(N, np.float32))
    M.apply(0, g)
    before = gpu_state(M)
    with pytest.raises(ga.GaError) as e:
        M.apply(2, g)
    assert e.value.status == ga.GA_ERR_WORKER and "worker 2" in str(e.value)
    with pytest.raises(ga.GaError) as e:
        M.run_schedule(np.array([0, 1, 5], np.uint32), ga.buffer_source([g]))
    assert e.value.status == ga.GA_ERR_WORKER
    with pytest.raises(ga.GaError) as e:
        M.diagnostics(0)                                        # m is not maintained in plain ASGD
    assert e.value.status == ga.GA_ERR_STATE
    with pytest.raises(ga.GaError):
        ga.ga_set_lr(M.ctx, 0.0)
    with pytest.raises(ga.GaError):
        ga.ga_set_beta_eps(ga.Master(8, 1).ctx, 0.999, 0.0)     # eps = 0 would make C = 0
    assert M.k == 1 and M.delays().tolist() == [1]
    for x, y in zip(before, gpu_state(M)):
        assert bits_equal(x, y) == 0
    M.run_schedule(np.zeros(0, np.uint32), ga.buffer_source([g]))   # empty schedule: no-op
    assert M.k == 1


def test_non_default_stream():
    N, W, seed = 70_001, 4, 3
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, 50, seed=seed)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        M = ga.Master(N, W, mode=ga.GA_MODE_GA, stream=s)
        M.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed))
        th = M.theta()
    s.synchronize()
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
    O.run_quadratic(sched, a, ts, seed)
    assert bits_equal(host(th), O.theta) == 0


@pytest.mark.parametrize("mode", [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_SA_STEP])
def test_untracked_modes_skip_m_and_snapshots(mode):
    # without gap tracking the non-GA modes move only theta, v and g (20 bytes per parameter)
    N, W, T = 9001, 4, 60
    bufs = ga_inputs.gradient_buffers(W, N, seed=2, std=0.1)
    sched = ga.ga_simulate_schedule(W, T, seed=2)
    M = ga.Master(N, W, mode=mode)
    M.run_schedule(sched, ga.buffer_source([dev(b) for b in bufs]))
    O = oracle.Master(N, W, mode, oracle.Hyper())
    O.run_buffers(sched, bufs)
    compare_masters(M, O, "untracked " + MODE_NAMES[mode], snaps=False, keep_m=False)
    th, v, m, sn = gpu_state(M)
    assert not m.any() and not sn.any()


@pytest.mark.parametrize("N", [1, 2, 3, 5, 64, 65])
def test_persistent_tiny_vectors(N):
    # fewer parameters than one 128-bit group, and the padding boundary of the state rows
    W, T, seed = 3, 40, 6
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    da = torch.zeros(((N + 3) // 4) * 4, dtype=torch.float32, device=DEV)[:N]
    dts = torch.zeros(((N + 3) // 4) * 4, dtype=torch.float32, device=DEV)[:N]
    da.copy_(dev(a))
    dts.copy_(dev(ts))
    for family, Oc, eta in [(ga.GA_FAMILY_MOMENTUM, oracle.Master, 0.1), (ga.GA_FAMILY_DANA, oracle.DanaMaster, 0.1),
                            (ga.GA_FAMILY_ADAM, oracle.AdamMaster, 0.01)]:
        M = ga.Master(N, W, eta=eta, mode=ga.GA_MODE_GA, family=family)
        M.run_schedule(sched, ga.quadratic_source(da, dts, seed))
        O = Oc(N, W, oracle.MODE_GA, oracle.Hyper(eta, 0.0 if family == ga.GA_FAMILY_ADAM else 0.9))
        O.run_quadratic(sched, a, ts, seed)
        assert bits_equal(host(M.theta()), O.theta) == 0, (N, family)
        for w in range(W):
            assert bits_equal(host(M.snapshot(w)), O.snaps[w]) == 0


@pytest.mark.parametrize("mode", [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_SA_STEP, ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE],
                         ids=["asgd", "sa", "sa_step", "ga", "ga_hinge"])
@pytest.mark.parametrize("path", ["persistent", "per_arrival", "buffers"])
def test_nesterov_form(mode, path):
    N, W, T, seed = 10_003, 6, 150, 12
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    M = ga.Master(N, W, eta=0.05, mode=mode, nesterov=True, track_gap=True)
    O = oracle.Master(N, W, mode, oracle.Hyper(0.05, 0.9), nesterov=True, track_gap=True)
    if path == "buffers":
        bufs = ga_inputs.gradient_buffers(W, N, seed, 0.2)
        M.run_schedule(sched, ga.buffer_source([dev(b) for b in bufs]))
        O.run_buffers(sched, bufs)
    else:
        g = torch.empty(N, dtype=torch.float32, device=DEV)
        M.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed, 0.01, path == "persistent", g))
        O.run_quadratic(sched, a, ts, seed)
    compare_masters(M, O, "nesterov %s %s" % (MODE_NAMES[mode], path))


def test_nesterov_layerwise_and_errors():
    N, W, T, seed = 5000, 4, 60, 3
    layers = [1000, 1500, 2500]
    bufs = ga_inputs.gradient_buffers(W, N, seed, 0.2)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    M = ga.Master(N, W, mode=ga.GA_MODE_GA, nesterov=True, layer_sizes=layers)
    M.run_schedule(sched, ga.buffer_source([dev(b) for b in bufs]))
    O = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), layers, nesterov=True)
    O.run_buffers(sched, bufs)
    compare_masters(M, O, "nesterov layer-wise")
    H = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), layers)
    H.run_buffers(sched, bufs)
    assert not np.array_equal(H.theta, O.theta)
    with pytest.raises(ga.GaError):
        ga.Master(N, W, family=ga.GA_FAMILY_DANA, nesterov=True)
    with pytest.raises(ga.GaError):
        ga.Master(N, W, family=ga.GA_FAMILY_ADAM, nesterov=True)
    assert torch.isfinite(M.theta()).all()


@pytest.mark.parametrize("mode", [ga.GA_MODE_GA, ga.GA_MODE_SA_STEP], ids=["ga", "sa_step"])
@pytest.mark.parametrize("path", ["persistent", "per_arrival", "buffers"])
def test_per_arrival_step_sizes(mode, path):
    # warm-up schedule (App. C.5): eta_k per arrival while eta_max stays at the peak value
    N, W, T, seed = 8_001, 8, 120, 4
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    lr = ga.ga_warmup_lr(0.1, W, 80, 0, T)
    M = ga.Master(N, W, eta=0.1, mode=mode, track_gap=True)
    O = oracle.Master(N, W, mode, oracle.Hyper(0.1, 0.9), track_gap=True)
    bufs = ga_inputs.gradient_buffers(W, N, seed, 0.2)
    g = torch.empty(N, dtype=torch.float32, device=DEV)
    if path == "buffers":
        src = ga.buffer_source([dev(b) for b in bufs])
    else:
        src = ga.quadratic_source(dev(a), dev(ts), seed, 0.01, path == "persistent", g)
    ga.ga_run_schedule_lr(M.ctx, sched[:50], src, lr[:50])
    ga.ga_run_schedule_lr(M.ctx, sched[50:], src, lr[50:])
    for k, w in enumerate(sched):
        w = int(w)
        O.hyper.eta_k = float(lr[k])
        O.apply(w, bufs[w] if path == "buffers" else oracle.quadratic_gradient(O.snaps[w], a, ts, seed, O.k + 1))
    compare_masters(M, O, "warm-up %s %s" % (MODE_NAMES[mode], path))
    with pytest.raises(ga.GaError):
        ga.ga_run_schedule_lr(M.ctx, sched[:2], src, np.array([0.1, -1.0], np.float32))


def test_many_workers_and_context_churn():
    # 1000 workers on a short vector; contexts created and destroyed repeatedly; two masters interleaved on two streams
    N, W, T, seed = 515, 1000, 3000, 2
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    da = torch.zeros(516, dtype=torch.float32, device=DEV)[:N]
    dts = torch.zeros(516, dtype=torch.float32, device=DEV)[:N]
    da.copy_(dev(a))
    dts.copy_(dev(ts))
    sched = ga.ga_simulate_schedule(W, T, ga.GA_DIST_LOGNORMAL, 1.0, seed)
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    M.run_schedule(sched, ga.quadratic_source(da, dts, seed))
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
    O.run_quadratic(sched, a, ts, seed)
    assert bits_equal(host(M.theta()), O.theta) == 0
    assert np.array_equal(M.delays(), np.array(O.tau_log, np.uint64)) and M.delays().max() > W
    for _ in range(200):
        X = ga.Master(64, 2, mode=ga.GA_MODE_GA)
        X.run_schedule(np.array([0, 1, 1], np.uint32), ga.quadratic_source(da[:64], dts[:64], 1))
        X.close()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    sched2 = ga.ga_simulate_schedule(4, 200, seed=5)
    with torch.cuda.stream(s1):
        A = ga.Master(N, 4, mode=ga.GA_MODE_GA, stream=s1)
    with torch.cuda.stream(s2):
        B = ga.Master(N, 4, mode=ga.GA_MODE_SA, stream=s2)
    for lo in range(0, 200, 25):
        with torch.cuda.stream(s1):
            A.run_schedule(sched2[lo:lo + 25], ga.quadratic_source(da, dts, 3))
        with torch.cuda.stream(s2):
            B.run_schedule(sched2[lo:lo + 25], ga.quadratic_source(da, dts, 4))
    with torch.cuda.stream(s1):
        ta = A.theta()
    with torch.cuda.stream(s2):
        tb = B.theta()
    torch.cuda.synchronize()
    OA = oracle.Master(N, 4, oracle.MODE_GA, oracle.Hyper())
    OA.run_quadratic(sched2, a, ts, 3)
    OB = oracle.Master(N, 4, oracle.MODE_SA, oracle.Hyper())
    OB.run_quadratic(sched2, a, ts, 4)
    assert bits_equal(host(ta), OA.theta) == 0 and bits_equal(host(tb), OB.theta) == 0
