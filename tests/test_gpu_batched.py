"""A queue of arrivals with gradient buffers applied by one launch (buffer source with `persistent` set):
parity with the oracle and bit identity with the per-arrival kernel (needs an MI355X)."""
import numpy as np
import pytest
import torch

import ga_inputs
import oracle
import paper_1909_10802_amd as ga
from gpu_util import DEV, MODE_NAMES, MODES, bits_equal, compare_masters, dev, gpu_state, host
from test_gpu_families import compare as compare_family, make_pair

pytestmark = pytest.mark.gpu


def make_bufs(n_bufs, N, seed, dtype):
    bufs = ga_inputs.gradient_buffers(n_bufs, N, seed=seed, std=0.3)
    if dtype == "bf16":
        bits = ga_inputs.f32_to_bf16_bits(bufs).reshape(n_bufs, N)
        return oracle.bf16_to_f32(bits).reshape(n_bufs, N), [dev(b.view(np.int16)).view(torch.bfloat16) for b in bits]
    return bufs, [dev(b) for b in bufs]


@pytest.mark.parametrize("mode", MODES, ids=[MODE_NAMES[m] for m in MODES])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 6, 20_011, 2_100_003])                 # two and four parameters per thread, ragged tails
def test_queue_equals_oracle_and_per_arrival_kernel(mode, dtype, N):
    W, T, n_bufs = 5, 40 if N > 10**6 else 150, 3
    ref, dbufs = make_bufs(n_bufs, N, 23, dtype)
    sched = ga.ga_simulate_schedule(W, T, seed=23)
    for pick in (ga.GA_PICK_BY_WORKER, ga.GA_PICK_BY_ARRIVAL):
        A = ga.Master(N, W, mode=mode, track_gap=True)
        A.run_schedule(sched[:T // 3], ga.buffer_source(dbufs, pick, persistent=True))   # the step counter carries over
        A.run_schedule(sched[T // 3:], ga.buffer_source(dbufs, pick, persistent=True))
        B = ga.Master(N, W, mode=mode, track_gap=True)
        B.run_schedule(sched, ga.buffer_source(dbufs, pick))
        for x, y, name in zip(gpu_state(A), gpu_state(B), ("theta", "v", "m", "snapshots")):
            assert bits_equal(x, y) == 0, name
        assert np.array_equal(A.delays(), B.delays()) and A.k == B.k
        if N < 10**6:
            O = oracle.Master(N, W, mode, oracle.Hyper(), track_gap=True)
            O.run_buffers(sched, np.ascontiguousarray(ref), pick_by_worker=(pick == ga.GA_PICK_BY_WORKER))
            compare_masters(A, O, "queue %s %s" % (MODE_NAMES[mode], dtype))
        A.close()
        B.close()


@pytest.mark.parametrize("family", [ga.GA_FAMILY_DANA, ga.GA_FAMILY_ADAM], ids=["dana", "adam"])
@pytest.mark.parametrize("mode", [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE], ids=["none", "sa", "ga", "ga_hinge"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N", [15_003, 2_100_003], ids=["two_per_thread", "four_per_thread"])
def test_queue_families(family, mode, dtype, N):
    W, T, n_bufs = 5, 120 if N < 10**6 else 16, 3
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    ref, dbufs = make_bufs(n_bufs, N, 9, dtype)
    sched = ga.ga_simulate_schedule(W, T, seed=9)
    M, O = make_pair(family, N, W, mode, eta)
    M.run_schedule(sched, ga.buffer_source(dbufs, ga.GA_PICK_BY_WORKER, persistent=True))
    O.run_buffers(sched, np.ascontiguousarray(ref))
    compare_family(M, O, "queue family %d mode %d %s" % (family, mode, dtype))


def test_queue_nesterov_and_step_sizes():
    N, W, T = 9_001, 4, 90
    ref, dbufs = make_bufs(2, N, 4, "f32")
    sched = ga.ga_simulate_schedule(W, T, seed=4)
    etas = ga.ga_warmup_lr(0.1, W, 60, 0, T)
    M = ga.Master(N, W, eta=0.1, mode=ga.GA_MODE_GA, nesterov=True)
    ga.ga_run_schedule_lr(M.ctx, sched, ga.buffer_source(dbufs, persistent=True), etas)
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper(0.1, 0.9), nesterov=True)
    for k, w in enumerate(sched):
        O.hyper.eta_k = float(etas[k])
        O.apply(int(w), ref[int(w) % 2])
    compare_masters(M, O, "queue nag + warm-up")


def test_queue_repeated_worker_and_more_than_one_table():
    N, W = 1003, 3
    ref, dbufs = make_bufs(3, N, 5, "f32")
    rng = np.random.default_rng(3)
    sched = np.concatenate([[0, 0, 0, 1, 1, 0, 2, 2, 2, 0], np.repeat(rng.integers(0, W, 4200), 2)]).astype(np.uint32)[:8192 + 33]
    M = ga.Master(N, W, mode=ga.GA_MODE_GA, eta=0.02)
    M.run_schedule(sched, ga.buffer_source(dbufs, persistent=True))
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper(0.02, 0.9))
    O.run_buffers(sched, ref)
    compare_masters(M, O, "queue repeats + two tables")


@pytest.mark.parametrize("mode", [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_SA_STEP])
def test_queue_without_tracking_leaves_m_and_snapshots_alone(mode):
    N, W, T = 5000, 3, 30
    ref, dbufs = make_bufs(3, N, 6, "f32")
    sched = ga.ga_simulate_schedule(W, T, seed=6)
    M = ga.Master(N, W, mode=mode, eta=0.01)
    marker = np.full(N, 7.5, np.float32)
    for w in range(W):
        ga.ga_put_snapshot(M.ctx, w, dev(marker))
    ga.ga_put_m(M.ctx, dev(marker))
    M.run_schedule(sched, ga.buffer_source(dbufs, persistent=True))
    O = oracle.Master(N, W, mode, oracle.Hyper(0.01, 0.9))
    O.run_buffers(sched, ref)
    assert bits_equal(host(M.theta()), O.theta) == 0 and bits_equal(host(M.v()), O.v) == 0
    assert np.array_equal(host(M.m()), marker)
    for w in range(W):
        assert np.array_equal(host(M.snapshot(w)), marker)


def test_queue_argument_errors():
    N, W = 1000, 2
    buf = torch.zeros(N + 4, dtype=torch.float32, device=DEV)
    M = ga.Master(N, W)
    with pytest.raises(ga.GaError) as e:
        M.run_schedule(np.zeros(3, np.uint32), ga.buffer_source([buf[1:N + 1]], persistent=True))
    assert e.value.status == ga.GA_ERR_ALIGN and M.k == 0
    M.run_schedule(np.zeros(3, np.uint32), ga.buffer_source([buf[1:N + 1]]))            # per arrival: any 4-byte alignment
    assert M.k == 3
    L = ga.Master(N, W, gap_scope=ga.GA_GAP_GLOBAL)
    with pytest.raises(ga.GaError) as e:
        L.run_schedule(np.zeros(3, np.uint32), ga.buffer_source([buf[:N]], persistent=True))
    assert e.value.status == ga.GA_ERR_ARG and L.k == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_apply_queue_equals_apply_one_by_one(dtype):
    # a queue given as (worker, gradient) pairs, longer than one table, against ga_apply per arrival and the oracle
    N, W, T = 4_099, 6, 300
    ref, dbufs = make_bufs(7, N, 31, dtype)
    rng = np.random.default_rng(8)
    workers = rng.integers(0, W, T).astype(np.uint32)
    which = rng.integers(0, 7, T)
    A = ga.Master(N, W, mode=ga.GA_MODE_GA, eta=0.05)
    A.apply_queue(workers[:100], [dbufs[b] for b in which[:100]])
    A.apply_queue(workers[100:], [dbufs[b] for b in which[100:]])
    A.apply_queue(workers[:0], [])                                     # an empty queue is a no-op
    B = ga.Master(N, W, mode=ga.GA_MODE_GA, eta=0.05)
    O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper(0.05, 0.9))
    for w, b in zip(workers, which):
        B.apply(int(w), dbufs[b])
        O.apply(int(w), ref[b])
    for x, y, name in zip(gpu_state(A), gpu_state(B), ("theta", "v", "m", "snapshots")):
        assert bits_equal(x, y) == 0, name
    compare_masters(A, O, "apply_queue %s" % dtype)


@pytest.mark.parametrize("family", [ga.GA_FAMILY_DANA, ga.GA_FAMILY_ADAM], ids=["dana", "adam"])
def test_apply_queue_families_bfloat16_four_per_thread(family):
    # ga_apply_queue itself (worker, gradient pairs) with bfloat16 gradients, at a size where a thread owns four parameters
    N, W, T = 2_100_003, 4, 14
    eta = 0.1 if family == ga.GA_FAMILY_DANA else 0.01
    ref, dbufs = make_bufs(3, N, 41, "bf16")
    rng = np.random.default_rng(5)
    workers = rng.integers(0, W, T).astype(np.uint32)
    which = rng.integers(0, 3, T)
    M, O = make_pair(family, N, W, ga.GA_MODE_GA, eta)
    M.apply_queue(workers, [dbufs[b] for b in which])
    for w, b in zip(workers, which):
        O.apply(int(w), ref[b])
    compare_family(M, O, "apply_queue family %d bf16" % family)


def test_apply_queue_errors_change_nothing():
    N, W = 1000, 2
    buf = torch.zeros(N + 4, dtype=torch.float32, device=DEV)
    M = ga.Master(N, W)
    for workers, grads, status in [([0, 2], [buf[:N], buf[:N]], ga.GA_ERR_WORKER),
                                   ([0, 1], [buf[:N], buf[1:N + 1]], ga.GA_ERR_ALIGN)]:
        with pytest.raises(ga.GaError) as e:
            M.apply_queue(workers, grads)
        assert e.value.status == status and M.k == 0
    with pytest.raises(ga.GaError) as e:
        ga.ga_apply_queue(M.ctx, [0], [buf[:N]], grad_dtype=7)
    assert e.value.status == ga.GA_ERR_ARG
    L = ga.Master(N, W, layer_sizes=[400, 600])
    with pytest.raises(ga.GaError) as e:
        L.apply_queue([0], [buf[:N]])
    assert e.value.status == ga.GA_ERR_ARG and L.k == 0
    assert float(M.theta().abs().sum()) == 0.0
