"""Pins for the oracle's arrival schedule and delay bookkeeping (no GPU).

Delay bookkeeping: Alg. 3 / Alg. 5 (iter = [0]*W, tau_k = k - iter[i]).
Master order: FIFO over arrivals (App. C.1).
"""
import numpy as np

import oracle


def test_hand_made_time_table():
    # worker 0 finishes at 1, 2, 3, ...; worker 1 at 2.5, 5, ...; worker 2 at 0.5, 4.5, ...
    times = np.array([[1.0] * 8, [2.5] * 8, [0.5, 4.0, 4.0, 4.0, 4.0, 4.0, 4.0, 4.0]])
    sched = oracle.schedule_from_times(times, 7)
    #          t: .5  1  2  2.5 3  4  4.5
    assert sched.tolist() == [2, 0, 0, 1, 0, 0, 2]


def test_ties_go_to_lowest_worker_id():
    times = np.ones((4, 6))
    sched = oracle.schedule_from_times(times, 12)
    assert sched.tolist() == [0, 1, 2, 3] * 3


def test_round_robin_delays_closed_form():
    W, T = 5, 23
    sched = np.arange(T, dtype=np.uint32) % W
    tau, it = oracle.delays(W, sched)
    assert tau.tolist() == [min(k, W) for k in range(1, T + 1)]
    assert it.tolist() == [max(k for k in range(1, T + 1) if (k - 1) % W == w) for w in range(W)]


def test_delay_invariants_on_random_schedule():
    W, T = 16, 5000
    sched = oracle.simulate_schedule(W, T, oracle.DIST_EXP, 1.0, seed=11)
    tau, it = oracle.delays(W, sched)
    assert tau.min() >= 1
    last = np.zeros(W, dtype=np.int64)
    for k, (w, t) in enumerate(zip(sched, tau), start=1):
        assert k - last[w] == t
        last[w] = k
    assert np.array_equal(last.astype(np.uint64), it)
    # resuming from a checkpointed (k, iter) continues the same delay sequence
    tau_a, it_a = oracle.delays(W, sched[:1234])
    tau_b, it_b = oracle.delays(W, sched[1234:], k0=1234, iter_=it_a.copy())
    assert np.array_equal(np.concatenate([tau_a, tau_b]), tau)
    assert np.array_equal(it_b, it)


def test_exponential_times_and_memoryless_delay():
    n = 200_000
    t = np.array([oracle.iteration_time(oracle.DIST_EXP, 1.0, 5, w % 7, w // 7) for w in range(n)])
    assert abs(t.mean() - 1.0) < 5 / np.sqrt(n)
    assert abs(t.var() - 1.0) < 5 * np.sqrt(8.0 / n)
    assert abs((t > 1.0).mean() - np.exp(-1.0)) < 5 * np.sqrt(0.25 / n)
    # Exp(1) workers are memoryless: each arrival is a uniformly random worker,
    # so the delay is geometric with mean W ("tau scales linearly with N", Sec. 3.1)
    for W in (8, 32):
        T = 200_000
        sched = oracle.simulate_schedule(W, T, oracle.DIST_EXP, 1.0, seed=W)
        tau, _ = oracle.delays(W, sched)
        steady = tau[20 * W:].astype(np.float64)
        assert abs(steady.mean() - W) < 0.03 * W
        assert abs(steady.var() - W * (W - 1)) < 0.08 * W * (W - 1)
        counts = np.bincount(sched, minlength=W)
        assert np.all(np.abs(counts - T / W) < 6 * np.sqrt(T / W))


def test_lognormal_times():
    n = 100_000
    for sigma in (1.0, 1.5):
        t = np.array([oracle.iteration_time(oracle.DIST_LOGNORMAL, sigma, 9, 3, i) for i in range(n)])
        lt = np.log(t)
        assert abs(lt.mean()) < 5 * sigma / np.sqrt(n)
        assert abs(lt.std() - sigma) < 0.01 * sigma
        assert abs(np.median(t) - 1.0) < 0.02


def test_heterogeneous_worker_means():
    sigma, n = 1.5, 20_000
    means = []
    for w in range(4):
        t = np.array([oracle.iteration_time(oracle.DIST_HETERO, sigma, 21, w, i) for i in range(n)])
        mu = t.mean()
        means.append(mu)
        # times / mean are Exp(1): variance of the ratio is 1
        assert abs((t / mu).var() - 1.0) < 0.1
    assert len({round(m, 3) for m in means}) == 4
    lm = np.log([np.mean([oracle.iteration_time(oracle.DIST_HETERO, sigma, 21, w, i) for i in range(400)])
                 for w in range(300)])
    assert abs(lm.std() - sigma) < 0.2


def test_schedule_is_counter_based():
    # a longer simulation has the shorter one as its prefix; finish times ascend
    s1, t1 = oracle.simulate_schedule(12, 500, oracle.DIST_LOGNORMAL, 1.0, seed=4, with_times=True)
    s2, t2 = oracle.simulate_schedule(12, 2000, oracle.DIST_LOGNORMAL, 1.0, seed=4, with_times=True)
    assert np.array_equal(s1, s2[:500]) and np.array_equal(t1, t2[:500])
    assert np.all(np.diff(t2) >= 0)
    # finish time of a worker's n-th arrival = sum of its first n iteration times
    w = int(s2[0])
    ks = np.nonzero(s2 == w)[0]
    acc = 0.0
    for n, k in enumerate(ks[:20]):
        acc += oracle.iteration_time(oracle.DIST_LOGNORMAL, 1.0, 4, w, n)
        assert t2[k] == acc
    assert not np.array_equal(s2, oracle.simulate_schedule(12, 2000, oracle.DIST_LOGNORMAL, 1.0, seed=5))
