"""GPU-vs-oracle parity of the layer-wise and global Gap (Eq. 4, Def. 1) (needs an MI355X)."""
import gc

import numpy as np
import pytest
import torch

import ga_inputs
import oracle
import paper_1909_10802_amd as ga
from gpu_util import DEV, RTOL_TRAJ_L2, assert_step_close, bits_equal, dev, gpu_state, host, load_state, rel_l2

pytestmark = pytest.mark.gpu

LAYERS = [1, 7, 32, 3, 8192 + 5, 20_000, 2, 8192, 4099]          # 40,533 parameters, odd boundaries


def check(M, O, what):
    th, v, m, sn = gpu_state(M)
    assert_step_close(th, O.theta, what + " theta")
    assert_step_close(v, O.v, what + " v")
    assert_step_close(m, O.m, what + " m")
    assert_step_close(sn, O.snaps, what + " snapshots")
    assert_step_close(M.layer_gaps(), O.last_gaps, what + " layer gaps")
    assert M.k == O.k and np.array_equal(M.delays(), np.array(O.tau_log, np.uint64))
    return bits_equal(th, O.theta)


@pytest.mark.parametrize("mode", [ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE], ids=["ga", "ga_hinge"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("offset", [0, 1])
def test_single_step_layerwise(mode, dtype, offset):
    N, W = sum(LAYERS), 3
    theta, v, m, snaps = ga_inputs.random_state(N, W, seed=3)
    g32 = (0.3 * ga_inputs.rng(3, 7).standard_normal(N + 4)).astype(np.float32)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(g32)
        g_ref = oracle.bf16_to_f32(bits)[offset:offset + N]
        g_dev = dev(bits.view(np.int16)).view(torch.bfloat16)[offset:offset + N]
    else:
        g_ref, g_dev = g32[offset:offset + N], dev(g32)[offset:offset + N]
    it = np.array([30, 22, 9], np.uint64)
    M = ga.Master(N, W, mode=mode, layer_sizes=LAYERS)
    load_state(M, theta, v, m, snaps, 30, it)
    M.apply(1, g_dev)
    O = oracle.LayerwiseMaster(N, W, mode, oracle.Hyper(), LAYERS)
    O.theta[:], O.v[:], O.m[:], O.snaps[:], O.k, O.iter[:] = theta, v, m, snaps, 30, it
    O.apply(1, np.ascontiguousarray(g_ref))
    assert check(M, O, "layer-wise single step") == 0


@pytest.mark.parametrize("scope", ["layer", "global"])
@pytest.mark.parametrize("mode", [ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE], ids=["ga", "ga_hinge"])
def test_trajectory_layerwise(scope, mode):
    N, W, T, seed = sum(LAYERS), 6, 150, 7
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    if scope == "layer":
        M = ga.Master(N, W, mode=mode, layer_sizes=LAYERS)
        O = oracle.LayerwiseMaster(N, W, mode, oracle.Hyper(), LAYERS)
    else:
        M = ga.Master(N, W, mode=mode, gap_scope=ga.GA_GAP_GLOBAL)
        O = oracle.LayerwiseMaster(N, W, mode, oracle.Hyper(), None)
    g = torch.empty(N, dtype=torch.float32, device=DEV)
    M.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed, 0.01, False, g))
    O.run_quadratic(sched, a, ts, seed)
    mism = check(M, O, "%s trajectory" % scope)
    assert rel_l2(host(M.theta()), O.theta) <= RTOL_TRAJ_L2
    print("%s Gap, mode %d: theta bit mismatches %d of %d" % (scope, mode, mism, N))


def test_layers_of_one_parameter_equal_parameter_wise_kernel():
    N, W, T, seed = 3000, 4, 60, 2
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T, seed=seed)
    g = torch.empty(N, dtype=torch.float32, device=DEV)
    A = ga.Master(N, W, mode=ga.GA_MODE_GA, layer_sizes=np.ones(N, np.uint64))
    B = ga.Master(N, W, mode=ga.GA_MODE_GA)
    A.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed, 0.01, False, g))
    B.run_schedule(sched, ga.quadratic_source(dev(a), dev(ts), seed, 0.01, False, g))
    assert bits_equal(host(A.theta()), host(B.theta())) == 0


def test_layerwise_argument_errors():
    ws = torch.empty(1 << 22, dtype=torch.uint8, device=DEV)
    bad = [dict(layer_sizes=[50, 49]), dict(layer_sizes=[100, 0]), dict(layer_sizes=[60, 60]),
           dict(gap_scope=ga.GA_GAP_LAYER), dict(gap_scope=5),
           dict(layer_sizes=[100], mode=ga.GA_MODE_SA), dict(layer_sizes=[100], family=ga.GA_FAMILY_DANA)]
    for kw in bad:
        cfg = ga.ga_config_init(N=100, n_workers=2, **kw)
        assert ga.ga_workspace_bytes_ex(cfg) == 0 or "mode" in kw or "family" in kw
        with pytest.raises(ga.GaError) as e:
            ga.ga_create_ex(cfg, ws)
        assert e.value.status == ga.GA_ERR_ARG, kw
    P = ga.Master(100, 2)
    with pytest.raises(ga.GaError) as e:
        ga.ga_get_layer_gaps(P.ctx, 1)
    assert e.value.status == ga.GA_ERR_STATE
    L = ga.Master(100, 2, layer_sizes=[40, 60])
    with pytest.raises(ga.GaError) as e:
        L.layer_gaps()                                            # no arrival yet
    assert e.value.status == ga.GA_ERR_STATE
    with pytest.raises(ga.GaError) as e:
        L.run_schedule(np.zeros(2, np.uint32), ga.quadratic_source(dev(np.ones(100, np.float32)),
                                                                    dev(np.ones(100, np.float32)), 1))
    assert e.value.status == ga.GA_ERR_ARG                        # no persistent kernel with a layer-wise Gap


def test_resnet50_size_161_layers():
    # cfg3's parameter vector and its 161 tensors; the oracle follows the whole vector (norms couple the
    # parameters of a layer), so fewer workers and arrivals than the benchmark
    cfg = ga_inputs.WORKLOADS["cfg3"]
    N, seed, W, T = cfg["N"], cfg["seed"], 8, 20
    sizes = ga_inputs.tensor_sizes(N, cfg["n_tensors"], seed)
    bufs = ga_inputs.device_gradient_buffers(W, N, seed, cfg["grad_std"], "f32", DEV)
    ref = np.stack([host(b) for b in bufs])
    sched = ga.ga_simulate_schedule(W, T, ga.GA_DIST_EXP, 1.0, seed)
    M = ga.Master(N, W, mode=ga.GA_MODE_GA, layer_sizes=sizes)
    M.run_schedule(sched, ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER))
    O = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), sizes)
    O.run_buffers(sched, ref)
    theta = host(M.theta())
    assert rel_l2(theta, O.theta) <= RTOL_TRAJ_L2
    assert_step_close(theta, O.theta, "theta")
    assert_step_close(host(M.m()), O.m, "m")
    assert_step_close(M.layer_gaps(), O.last_gaps, "layer gaps")
    print("161 layers: theta bit mismatches %d of %d; gaps %.3f..%.3f"
          % (bits_equal(theta, O.theta), N, O.last_gaps.min(), O.last_gaps.max()))
    del M, bufs
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("scope", ["layer", "global"])
@pytest.mark.parametrize("nesterov", [False, True], ids=["heavy_ball", "nag"])
def test_sums_prepared_by_the_previous_update_equal_the_separate_pass(scope, nesterov):
    # Inside one ga_run_schedule call the update pass of an arrival also forms the norms of the next
    # one (the next worker is known); arrival by arrival, a separate reduction pass forms them.  Both
    # must give the same bits, also when a worker arrives twice in a row, and both must match the oracle.
    N, W, seed = sum(LAYERS), 4, 13
    kw = dict(layer_sizes=LAYERS) if scope == "layer" else dict(gap_scope=ga.GA_GAP_GLOBAL)
    bufs = ga_inputs.gradient_buffers(W, N + 1, seed=seed, std=0.3)
    dbufs = [dev(b)[1:] for b in bufs]                                  # 4-byte aligned only
    sched = np.array([0, 1, 1, 1, 2, 0, 0, 3, 2, 2, 1, 3, 3, 0, 2, 1, 1, 0], dtype=np.uint32)
    src = ga.buffer_source(dbufs, ga.GA_PICK_BY_WORKER)
    A = ga.Master(N, W, mode=ga.GA_MODE_GA, nesterov=nesterov, **kw)
    A.run_schedule(sched[:11], src)                                     # two calls: nothing is carried across
    A.run_schedule(sched[11:], src)
    B = ga.Master(N, W, mode=ga.GA_MODE_GA, nesterov=nesterov, **kw)
    for w in sched:
        B.apply(int(w), dbufs[int(w)])
    O = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), LAYERS if scope == "layer" else None,
                               nesterov=nesterov)
    O.run_buffers(sched, np.ascontiguousarray(bufs[:, 1:]))
    sa, sb = gpu_state(A), gpu_state(B)
    for x, y, name in zip(sa, sb, ("theta", "v", "m", "snapshots")):
        assert bits_equal(x, y) == 0, name
    assert bits_equal(A.layer_gaps(), B.layer_gaps()) == 0
    check(A, O, "%s look-ahead" % scope)


def test_state_written_between_calls_is_seen_by_the_next_arrival():
    # the norms prepared for a following arrival never outlive a call: putting a new m or theta
    # between two calls changes the next Gap exactly as the oracle says
    N, W, seed = sum(LAYERS), 3, 17
    bufs = ga_inputs.gradient_buffers(W, N, seed=seed, std=0.3)
    dbufs = [dev(b) for b in bufs]
    src = ga.buffer_source(dbufs, ga.GA_PICK_BY_WORKER)
    M = ga.Master(N, W, mode=ga.GA_MODE_GA, layer_sizes=LAYERS)
    O = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), LAYERS)
    first, second = np.array([0, 1, 2, 0], np.uint32), np.array([1, 1, 2], np.uint32)
    M.run_schedule(first, src)
    O.run_buffers(first, bufs)
    new_m = (4.0 * O.m + 1e-3).astype(np.float32)
    new_theta = (O.theta + 0.25).astype(np.float32)
    O.m[:], O.theta[:] = new_m, new_theta
    ga.ga_put_m(M.ctx, dev(new_m))
    ga.ga_put_theta(M.ctx, dev(new_theta))
    M.run_schedule(second, src)
    O.run_buffers(second, bufs)
    assert check(M, O, "after put") == 0


@pytest.mark.parametrize("scope", ["layer", "global"])
def test_beyond_the_cache_resident_size(scope):
    # past 30 M parameters v is streamed in the update pass (another instantiation); whole vector against the oracle
    N, W, T, seed = 33_000_003, 3, 7, 15
    sizes = ga_inputs.tensor_sizes(N, 40, seed)
    bufs = ga_inputs.device_gradient_buffers(2, N, seed, 0.3, "f32", DEV)
    ref = np.stack([host(b) for b in bufs])
    sched = np.array([0, 1, 1, 2, 0, 2, 1], dtype=np.uint32)
    if scope == "layer":
        M = ga.Master(N, W, mode=ga.GA_MODE_GA, layer_sizes=sizes)
        O = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), sizes)
    else:
        M = ga.Master(N, W, mode=ga.GA_MODE_GA, gap_scope=ga.GA_GAP_GLOBAL)
        O = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), None)
    M.run_schedule(sched, ga.buffer_source(bufs, ga.GA_PICK_BY_WORKER))
    O.run_buffers(sched, ref)
    theta = host(M.theta())
    assert rel_l2(theta, O.theta) <= RTOL_TRAJ_L2
    assert_step_close(theta, O.theta, "theta")
    assert_step_close(host(M.v()), O.v, "v")
    assert_step_close(host(M.m()), O.m, "m")
    assert_step_close(M.layer_gaps(), O.last_gaps, "layer gaps")
    del M, bufs
    gc.collect()
    torch.cuda.empty_cache()
