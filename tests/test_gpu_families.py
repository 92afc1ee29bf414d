"""GPU-vs-oracle parity of the DANA (Alg. 6-8) and Adam (Alg. 9-11) masters (needs an MI355X)."""
import gc

import numpy as np
import pytest
import torch

import ga_inputs
import oracle
import paper_1909_10802_amd as ga
from gpu_util import DEV, RTOL_TRAJ_L2, assert_step_close, bits_equal, dev, host, rel_l2

pytestmark = pytest.mark.gpu

PENALTIES = [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE]
NAMES = {0: "none", 1: "sa", 3: "ga", 4: "ga_hinge"}
FAMILIES = [ga.GA_FAMILY_DANA, ga.GA_FAMILY_ADAM]
FNAME = {1: "dana", 2: "adam"}


def make_pair(family, N, W, mode, eta, track=True, **kw):
    M = ga.Master(N, W, eta=eta, gamma=0.9, mode=mode, family=family, track_gap=track, **kw)
    if family == ga.GA_FAMILY_DANA:
        O = oracle.DanaMaster(N, W, mode, oracle.Hyper(eta, 0.9), track_gap=track)
    else:
        O = oracle.AdamMaster(N, W, mode, oracle.Hyper(eta, 0.0), track_gap=track)
    return M, O


def compare(M, O, what, keep_m=True, snaps=True, exact=True):
    torch.cuda.synchronize()
    th = host(M.theta())
    assert_step_close(th, O.theta, what + " theta")
    if M.family == ga.GA_FAMILY_DANA:
        assert_step_close(host(M.v()), O.vsum, what + " vsum")
        for w in range(M.W):
            assert_step_close(host(M.array(ga.GA_ARR_WORKER_V, w)), O.vw[w], what + " v_%d" % w)
    else:
        assert_step_close(host(M.v()), O.m1, what + " m1")
        assert_step_close(host(M.array(ga.GA_ARR_ADAM_V2)), O.v2, what + " v2")
    if keep_m:
        assert_step_close(host(M.m()), O.m, what + " m")
    if snaps:
        for w in range(M.W):
            assert_step_close(host(M.snapshot(w)), O.snaps[w], what + " snapshot %d" % w)
    assert M.k == O.k and np.array_equal(M.iter(), O.iter)
    assert np.array_equal(M.delays(), np.array(O.tau_log, np.uint64))
    if exact:
        assert bits_equal(th, O.theta) == 0, what + ": theta not bit-identical"


def load(M, O):
    """Copy the oracle's state into the GPU master."""
    ga.ga_put_theta(M.ctx, dev(O.theta))
    ga.ga_put_m(M.ctx, dev(O.m))
    for w in range(M.W):
        ga.ga_put_snapshot(M.ctx, w, dev(O.snaps[w]))
    if M.family == ga.GA_FAMILY_DANA:
        ga.ga_put_v(M.ctx, dev(O.vsum))
        for w in range(M.W):
            ga.ga_put_array(M.ctx, ga.GA_ARR_WORKER_V, w, dev(O.vw[w]))
    else:
        ga.ga_put_v(M.ctx, dev(O.m1))
        ga.ga_put_array(M.ctx, ga.GA_ARR_ADAM_V2, 0, dev(O.v2))
    ga.ga_set_bookkeeping(M.ctx, O.k, O.iter)


@pytest.mark.parametrize("family", FAMILIES, ids=["dana", "adam"])
@pytest.mark.parametrize("mode", PENALTIES, ids=[NAMES[m] for m in PENALTIES])
@pytest.mark.parametrize("N", [1, 3, 5, 1024, 2048 + 7, 100_003])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_step(family, mode, N, dtype):
    W, k, tau = 3, 41, 6
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    M, O = make_pair(family, N, W, mode, eta)
    theta, v, m, snaps = ga_inputs.random_state(N, W, seed=N + family)
    r = ga_inputs.rng(N, 11)
    O.theta[:], O.m[:], O.snaps[:] = theta, m, snaps
    if family == ga.GA_FAMILY_DANA:
        O.vw[:] = (0.1 * r.standard_normal((W, N))).astype(np.float32)
        O.vsum[:] = O.vw.sum(0)
    else:
        O.m1[:] = v
        O.v2[:] = (0.01 * r.random(N)).astype(np.float32)
    O.k, O.iter[:] = k - 1, [k - 1, k - tau, 2]
    load(M, O)
    g32 = (0.3 * r.standard_normal(N)).astype(np.float32)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(g32)
        g_ref, g_dev = oracle.bf16_to_f32(bits), dev(bits.view(np.int16)).view(torch.bfloat16)
    else:
        g_ref, g_dev = g32, dev(g32)
    M.apply(1, g_dev)
    assert O.apply(1, g_ref) == tau
    compare(M, O, "%s %s N=%d %s" % (FNAME[family], NAMES[mode], N, dtype))


@pytest.mark.parametrize("family", FAMILIES, ids=["dana", "adam"])
@pytest.mark.parametrize("mode", PENALTIES, ids=[NAMES[m] for m in PENALTIES])
@pytest.mark.parametrize("persistent", [False, True], ids=["per_arrival", "persistent"])
def test_trajectory_quadratic(family, mode, persistent):
    N, W, T, seed = 20_003, 8, 200, 4
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    M, O = make_pair(family, N, W, mode, eta, track=False)
    scratch = torch.empty(N, dtype=torch.float32, device=DEV)
    src = ga.quadratic_source(dev(a), dev(ts), seed, 0.01, persistent, scratch)
    M.run_schedule(sched[:90], src)                       # two calls: the step counter and Adam's bias corrections carry over
    M.run_schedule(sched[90:], src)
    O.run_quadratic(sched, a, ts, seed)
    compare(M, O, "%s %s quadratic" % (FNAME[family], NAMES[mode]), keep_m=mode in (3, 4))
    assert rel_l2(host(M.theta()), O.theta) <= RTOL_TRAJ_L2


@pytest.mark.parametrize("family", FAMILIES, ids=["dana", "adam"])
def test_persistent_repeated_worker_and_chunks(family):
    N, W, seed = 1000 + 3, 3, 5
    eta = 0.05 if family == ga.GA_FAMILY_DANA else 0.01
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    rng = np.random.default_rng(2)
    sched = np.concatenate([[0, 0, 0, 1, 1, 0, 2, 2, 2, 0], np.repeat(rng.integers(0, W, 4200), 2)]).astype(np.uint32)[:8192 + 21]
    M, O = make_pair(family, N, W, ga.GA_MODE_GA, eta, track=False)
    M.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed))
    O.run_quadratic(sched, a, ts, seed)
    compare(M, O, "%s repeats + chunks" % FNAME[family])


@pytest.mark.parametrize("family", FAMILIES, ids=["dana", "adam"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_trajectory_buffers(family, dtype):
    N, W, T, n_bufs = 15_001, 5, 120, 3
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    bufs = ga_inputs.gradient_buffers(n_bufs, N, seed=9, std=0.3)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(bufs).reshape(n_bufs, N)
        ref, dbufs = oracle.bf16_to_f32(bits).reshape(n_bufs, N), [dev(b.view(np.int16)).view(torch.bfloat16) for b in bits]
    else:
        ref, dbufs = bufs, [dev(b) for b in bufs]
    sched = ga.ga_simulate_schedule(W, T, seed=9)
    for mode in PENALTIES:
        for track in (True, False):
            M, O = make_pair(family, N, W, mode, eta, track=track)
            M.run_schedule(sched, ga.buffer_source(dbufs, ga.GA_PICK_BY_ARRIVAL))
            O.run_buffers(sched, ref, pick_by_worker=False)
            full = track or mode in (3, 4)
            compare(M, O, "%s %s buffers" % (FNAME[family], NAMES[mode]), keep_m=full, snaps=full)


def test_single_worker_penalties_coincide_adam():
    N, T, seed = 4000, 30, 2
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    outs = []
    for mode in PENALTIES:
        M = ga.Master(N, 1, eta=0.01, mode=mode, family=ga.GA_FAMILY_ADAM)
        g = torch.empty(N, dtype=torch.float32, device=DEV)
        M.run_schedule(np.zeros(T, np.uint32), ga.quadratic_source(dev(a), dev(ts), seed, 0.01, False, g))
        outs.append(host(M.theta()))
    assert all(bits_equal(o, outs[0]) == 0 for o in outs[1:])


def test_family_argument_errors():
    ws = torch.empty(1 << 22, dtype=torch.uint8, device=DEV)
    for kw in (dict(family=7), dict(family=ga.GA_FAMILY_DANA, mode=ga.GA_MODE_SA_STEP),
               dict(family=ga.GA_FAMILY_ADAM, adam_beta1=1.0), dict(family=ga.GA_FAMILY_ADAM, adam_eps=0.0),
               dict(beta=1.0), dict(eps=0.0)):
        with pytest.raises(ga.GaError) as e:
            ga.ga_create_ex(ga.ga_config_init(N=100, n_workers=2, **kw), ws)
        assert e.value.status == ga.GA_ERR_ARG, kw
    M = ga.Master(100, 2, family=ga.GA_FAMILY_ADAM)
    with pytest.raises(ga.GaError):
        M.array(ga.GA_ARR_WORKER_V, 0)                     # Adam has no per-worker momenta
    D = ga.Master(100, 2, family=ga.GA_FAMILY_DANA)
    with pytest.raises(ga.GaError) as e:
        D.array(ga.GA_ARR_WORKER_V, 2)
    assert e.value.status == ga.GA_ERR_WORKER
    # DANA: every worker's snapshot and momentum are a tiled pair (tiles of 8192 floats) instead of one row of 128
    assert ga.ga_workspace_bytes_ex(ga.ga_config_init(N=128, n_workers=4, family=ga.GA_FAMILY_DANA)) \
        - ga.ga_workspace_bytes(128, 4) == 4 * (2 * 8192 - 128) * 4
    # Adam's second moment is a fourth array in the tile structure of theta, m1, m (tiles of 8192 floats)
    assert ga.ga_workspace_bytes_ex(ga.ga_config_init(N=128, n_workers=4, family=ga.GA_FAMILY_ADAM)) \
        - ga.ga_workspace_bytes(128, 4) == 8192 * 4


@pytest.mark.parametrize("family", FAMILIES, ids=["dana", "adam"])
def test_resnet50_size_sampled(family):
    # the cfg3 workload (N = 25.6 M, 64 workers, 64 float gradient buffers, 2000 arrivals), GA penalty
    cfg = ga_inputs.WORKLOADS["cfg3"]
    N, W, T, seed = cfg["N"], cfg["W"], 600, cfg["seed"]
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    idx = ga_inputs.sample_indices(N, 12000, seed)
    idx_dev = torch.from_numpy(idx.astype(np.int64)).to(DEV)
    bufs = ga_inputs.device_gradient_buffers(cfg["n_bufs"], N, seed, cfg["grad_std"], "f32", DEV)
    bufs_s = np.stack([host(b[idx_dev]) for b in bufs])
    sched = ga.ga_simulate_schedule(W, T, ga.GA_DIST_EXP, 1.0, seed)
    M = ga.Master(N, W, eta=eta, gamma=0.9, mode=ga.GA_MODE_GA, family=family)
    M.run_schedule(sched, ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER))
    if family == ga.GA_FAMILY_DANA:
        O = oracle.DanaMaster(idx.size, W, oracle.MODE_GA, oracle.Hyper(eta, 0.9))
    else:
        O = oracle.AdamMaster(idx.size, W, oracle.MODE_GA, oracle.Hyper(eta, 0.0))
    O.run_buffers(sched, bufs_s, pick_by_worker=True)
    theta = host(M.theta()[idx_dev])
    assert rel_l2(theta, O.theta) <= RTOL_TRAJ_L2
    assert_step_close(theta, O.theta, "theta")
    assert_step_close(host(M.m()[idx_dev]), O.m, "m")
    for w in (0, 17, 63):
        assert_step_close(host(M.snapshot(w)[idx_dev]), O.snaps[w], "snapshot %d" % w)
    assert np.array_equal(M.delays(), np.array(O.tau_log, np.uint64))
    print("%s cfg3-size: %d sampled, theta bit mismatches %d" % (FNAME[family], idx.size, bits_equal(theta, O.theta)))
    del M, bufs
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("family", [ga.GA_FAMILY_MOMENTUM, ga.GA_FAMILY_DANA, ga.GA_FAMILY_ADAM], ids=["momentum", "dana", "adam"])
def test_export_import_state_resumes_bit_identically(family):
    N, W, T, seed = 30_001, 5, 140, 8
    eta = 0.01 if family == ga.GA_FAMILY_ADAM else 0.1
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    src = ga.quadratic_source(dev(a), dev(ts), seed)
    A = ga.Master(N, W, eta=eta, mode=ga.GA_MODE_GA, family=family)
    A.run_schedule(sched, src)
    B = ga.Master(N, W, eta=eta, mode=ga.GA_MODE_GA, family=family)
    B.run_schedule(sched[:60], src)
    ckpt = torch.empty(ga.ga_state_bytes(B.ctx), dtype=torch.uint8, device=DEV)
    k, it = ga.ga_export_state(B.ctx, W, ckpt)
    assert k == 60 and np.array_equal(it, B.iter())
    C2 = ga.Master(N, W, eta=eta, mode=ga.GA_MODE_GA, family=family)
    ga.ga_import_state(C2.ctx, ckpt, k, it)
    C2.run_schedule(sched[60:], src)
    assert bits_equal(host(A.theta()), host(C2.theta())) == 0 and bits_equal(host(A.m()), host(C2.m())) == 0
    for w in range(W):
        assert bits_equal(host(A.snapshot(w)), host(C2.snapshot(w))) == 0
    assert C2.k == A.k and np.array_equal(C2.iter(), A.iter())
    other = ga.Master(N + 8192, W, eta=eta, mode=ga.GA_MODE_GA, family=family)     # one more tile of every tiled array
    with pytest.raises(ga.GaError) as e:
        ga.ga_import_state(other.ctx, ckpt, k, it)
    assert e.value.status == ga.GA_ERR_ARG
    with pytest.raises(ga.GaError):
        ga.ga_import_state(C2.ctx, ckpt, 3, np.full(W, 9, np.uint64))


@pytest.mark.parametrize("family", FAMILIES, ids=["dana", "adam"])
@pytest.mark.parametrize("N,dtype", [(33_000_003, "f32"), (33_000_003, "bf16"), (70_000_001, "bf16")],
                         ids=["33M-f32", "33M-bf16", "70M-bf16"])
def test_beyond_the_cache_resident_size_sampled(family, N, dtype):
    # past 30 M parameters only a leading part of the second state array stays in the memory-side cache, past
    # 63 M only a leading part of theta: the block-uniform paths of the fused kernel, float and bfloat16 gradients
    W, T, seed = 3, 12, 14
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    idx = ga_inputs.sample_indices(N, 8000, seed)
    idx_dev = torch.from_numpy(idx.astype(np.int64)).to(DEV)
    bufs = ga_inputs.device_gradient_buffers(2, N, seed, 0.3, dtype, DEV)
    bufs_s = np.stack([host(b[idx_dev].to(torch.float32)) for b in bufs])     # widening bfloat16 is exact
    sched = ga.ga_simulate_schedule(W, T, ga.GA_DIST_EXP, 1.0, seed)
    M = ga.Master(N, W, eta=eta, gamma=0.9, mode=ga.GA_MODE_GA, family=family)
    M.run_schedule(sched, ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER))
    if family == ga.GA_FAMILY_DANA:
        O = oracle.DanaMaster(idx.size, W, oracle.MODE_GA, oracle.Hyper(eta, 0.9))
    else:
        O = oracle.AdamMaster(idx.size, W, oracle.MODE_GA, oracle.Hyper(eta, 0.0))
    O.run_buffers(sched, bufs_s, pick_by_worker=True)
    theta = host(M.theta()[idx_dev])
    assert bits_equal(theta, O.theta) == 0
    assert_step_close(host(M.v()[idx_dev]), O.vsum if family == ga.GA_FAMILY_DANA else O.m1, "x")
    assert_step_close(host(M.m()[idx_dev]), O.m, "m")
    for w in range(W):
        assert_step_close(host(M.snapshot(w)[idx_dev]), O.snaps[w], "snapshot %d" % w)
    del M, bufs
    gc.collect()
    torch.cuda.empty_cache()
