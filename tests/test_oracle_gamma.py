"""Pins for the gamma execution-time model (Alg. 12, 13) and the speed-up simulation (App. D); no GPU."""
import os

import numpy as np
from scipy import stats

import oracle
import paper_1909_10802_amd as ga

GOLD = dict(l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "gamma_model_app_c3_d.txt"))
            if l[0] not in "#\n")
MEAN = float(GOLD["mean"])
LIMIT = MEAN * float(GOLD["threshold_factor"])


def test_gamma_variates_follow_the_gamma_law():
    for alpha, scale in [(100.0, 1.28), (1.0 / 0.36, 46.08), (1.0, 2.0)]:
        x = np.array([oracle.gamma_draw(alpha, scale, 7, i) for i in range(100_000)])
        assert stats.kstest(x, stats.gamma(a=alpha, scale=scale).cdf).pvalue > 1e-3
        assert abs(x.mean() - alpha * scale) < 5 * np.sqrt(alpha) * scale / np.sqrt(x.size)
        assert abs(x.var() / (alpha * scale ** 2) - 1) < 0.03


def test_printed_tail_probabilities():
    # heterogeneous (Alg. 13): pooled over machines the tail is the printed 27.9 %
    t = np.array([oracle.iteration_time_gamma(oracle.DIST_GAMMA_HETERO, 3, w, n, MEAN, 0.6, 0.1)
                  for w in range(4000) for n in range(25)])
    assert abs((t >= LIMIT).mean() - float(GOLD["tail_heterogeneous"])) < 0.015
    assert abs(t.mean() / MEAN - 1) < 0.03
    # homogeneous (Alg. 12): times are G(100, q/100); for q at its mean the tail is the printed 1 %
    assert abs(stats.gamma.sf(LIMIT, a=100, scale=MEAN / 100) - float(GOLD["tail_homogeneous"])) < 0.002
    # and the simulated times of a run follow G(100, q/100) for that run's q
    for seed in (1, 2, 3):
        t = np.array([oracle.iteration_time_gamma(oracle.DIST_GAMMA_HOMO, seed, w, n, MEAN, 0.1, 0.1)
                      for w in range(20) for n in range(2000)])
        q = t.mean()
        assert abs(q / MEAN - 1) < 0.4                                       # q ~ G(100, 1.28): cv 0.1
        assert stats.kstest(t, stats.gamma(a=100, scale=q / 100).cdf).pvalue > 1e-4
        assert abs((t >= 1.25 * q).mean() - stats.gamma.sf(125, a=100)) < 0.004


def test_speedup_matches_the_printed_ratios():
    # homogeneous: SSGD pays the maximum of W gamma times per batch; at 32 workers ASGD is ~21 % faster
    ratios = []
    for seed in range(4):
        a, s = oracle.speedup_times(32, 5000, oracle.DIST_GAMMA_HOMO, seed, MEAN, 0.1, 0.1)
        ratios.append(s / a)
    assert abs(np.mean(ratios) - float(GOLD["speedup_ratio_homogeneous_max"])) < 0.02
    # fewer workers: smaller gain; one worker: none
    a, s = oracle.speedup_times(4, 5000, oracle.DIST_GAMMA_HOMO, 0, MEAN, 0.1, 0.1)
    assert 1.05 < s / a < 1.15
    a, s = oracle.speedup_times(1, 2000, oracle.DIST_GAMMA_HOMO, 0, MEAN, 0.1, 0.1)
    assert abs(s / a - 1) < 1e-12
    # heterogeneous: the slowest machine sets the SSGD pace; the gain grows with W and reaches ~6x
    het = {}
    for W in (8, 32, 128):
        r = []
        for seed in range(12):
            a, s = oracle.speedup_times(W, 400, oracle.DIST_GAMMA_HETERO, seed, MEAN, 0.6, 0.1)
            r.append(s / a)
        het[W] = float(np.mean(r))
    assert het[8] < het[32] < het[128]
    assert 0.75 * float(GOLD["speedup_ratio_heterogeneous_max"]) < het[128] < 1.35 * float(GOLD["speedup_ratio_heterogeneous_max"])


def test_library_time_models_match_the_oracle_bit_for_bit():
    for dist, vm in [(ga.GA_DIST_GAMMA_HOMO, 0.1), (ga.GA_DIST_GAMMA_HETERO, 0.6)]:
        model = ga.time_model(dist, mean=MEAN, v_mach=vm, v_task=0.1)
        for W, T, seed in [(1, 40, 0), (8, 2000, 3), (64, 5000, 2**35 + 1)]:
            mine, tm = ga.ga_simulate_schedule_ex(W, T, model, seed, with_times=True)
            ref, tr = oracle.simulate_schedule_gamma(W, T, dist, seed, MEAN, vm, 0.1, with_times=True)
            assert np.array_equal(mine, ref) and np.array_equal(tm, tr)
        a, s = ga.ga_simulate_speedup(16, 300, model, 5)
        assert (a, s) == oracle.speedup_times(16, 300, dist, 5, MEAN, vm, 0.1)
    for dist, sigma in [(ga.GA_DIST_EXP, 1.0), (ga.GA_DIST_LOGNORMAL, 1.0), (ga.GA_DIST_HETERO, 1.5)]:
        mine, tm = ga.ga_simulate_schedule_ex(16, 1000, ga.time_model(dist, sigma), 9, with_times=True)
        ref, tr = oracle.simulate_schedule(16, 1000, dist, sigma, 9, with_times=True)
        assert np.array_equal(mine, ref) and np.array_equal(tm, tr)
    for bad in (ga.time_model(9), ga.time_model(ga.GA_DIST_GAMMA_HOMO, mean=0.0), ga.time_model(ga.GA_DIST_GAMMA_HETERO, v_mach=2.0)):
        try:
            ga.ga_simulate_schedule_ex(4, 10, bad, 0)
            raise AssertionError("accepted a bad time model")
        except ga.GaError as e:
            assert e.status == ga.GA_ERR_ARG
