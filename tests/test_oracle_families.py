"""Pins for the oracle's DANA (Alg. 6-8) and Adam (Alg. 9-11) masters (no GPU)."""
import numpy as np
import pytest
import torch

import ga_inputs
import oracle
from oracle import (MODE_ASGD, MODE_GA, MODE_GA_HINGE, MODE_SA, AdamMaster, DanaMaster, Hyper, Master)

PENALTIES = [MODE_ASGD, MODE_SA, MODE_GA, MODE_GA_HINGE]


def quad_inputs(N, seed, dtype):
    return ga_inputs.curvatures(N, seed).astype(dtype), ga_inputs.optimum(N, seed).astype(dtype)


# ------------------------------------------------------------------ DANA
@pytest.mark.parametrize("gamma", [0.9, 0.5])
def test_dana_single_worker_closed_form(gamma):
    # One worker, noise-free quadratic.  The worker holds the look-ahead s = theta - eta gamma v, so
    # g = a (e - eta gamma v) with e = theta - theta*;  v' = gamma v + g;  e' = e - eta v'.
    N, T, eta = 32, 150, 0.1
    a, ts = quad_inputs(N, 3, np.float64)
    D = DanaMaster(N, 1, MODE_ASGD, Hyper(eta, gamma, f32=False), np.float64)
    D.run_quadratic(np.zeros(T, np.uint32), a, ts, seed=0, sigma=0.0)
    for j in range(N):
        q = gamma - a[j] * eta * gamma
        A = np.array([[1 - eta * a[j], -eta * q], [a[j], q]])
        e, v = np.linalg.matrix_power(A, T) @ np.array([-ts[j], 0.0])
        assert abs(D.theta[j] - (ts[j] + e)) < 1e-12 and abs(D.vw[0, j] - v) < 1e-12
        assert abs(D.snaps[0, j] - (D.theta[j] - eta * gamma * v)) < 1e-15


@pytest.mark.parametrize("mode", PENALTIES)
def test_dana_without_momentum_is_the_plain_master(mode):
    # gamma = 0: v^i is the penalised gradient, the look-ahead equals theta (Alg. 6-8 reduce to Alg. 2/5/4)
    N, W, T = 500, 5, 120
    a, ts = quad_inputs(N, 7, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=7)
    D = DanaMaster(N, W, mode, Hyper(0.1, 0.0), np.float32)
    M = Master(N, W, mode, Hyper(0.1, 0.0), np.float32)
    D.run_quadratic(sched, a, ts, seed=5)
    M.run_quadratic(sched, a, ts, seed=5)
    assert np.array_equal(D.theta, M.theta) and np.array_equal(D.snaps, M.snaps)
    if mode in (MODE_GA, MODE_GA_HINGE):
        assert np.array_equal(D.m, M.m)
    assert D.tau_log == M.tau_log


def test_dana_momentum_sum_and_lookahead_invariants():
    N, W, T, eta, gamma = 64, 6, 300, 0.05, 0.9
    a, ts = quad_inputs(N, 2, np.float64)
    sched = oracle.simulate_schedule(W, T, seed=2)
    for mode in PENALTIES:
        D = DanaMaster(N, W, mode, Hyper(eta, gamma, f32=False), np.float64)
        for t, w in enumerate(sched):
            w = int(w)
            others = [D.vw[u].copy() for u in range(W) if u != w]
            D.apply(w, oracle.quadratic_gradient(D.snaps[w], a, ts, 3, D.k + 1, 0.01))
            assert np.allclose(D.vsum, D.vw.sum(0), rtol=1e-11, atol=1e-13)              # sum_j v^j
            assert np.allclose(D.snaps[w], D.theta - eta * gamma * D.vw.sum(0), rtol=1e-11, atol=1e-13)
            assert all(np.array_equal(x, D.vw[u]) for x, u in zip(others, [u for u in range(W) if u != w]))


def test_dana_constant_gradient_closed_forms():
    # Alg. 6, round robin, the same gradient c from everyone: after its n-th arrival a worker has
    # v^i = c (1 - gamma^n)/(1 - gamma); theta_K = -eta * sum of the momenta used.
    N, W, T, eta, gamma = 4, 3, 40, 0.1, 0.8
    c = np.array([1.0, -2.0, 0.5, 3.0])
    D = DanaMaster(N, W, MODE_ASGD, Hyper(eta, gamma, f32=False), np.float64)
    D.run_buffers((np.arange(T) % W).astype(np.uint32), c[None, :])
    used = 0.0
    for k in range(1, T + 1):
        n = (k - 1) // W + 1
        used += (1 - gamma ** n) / (1 - gamma)
    assert np.allclose(D.theta, -eta * c * used, rtol=1e-12)
    # Alg. 7: tau = W in steady state, so every momentum settles at (c / W)/(1 - gamma)
    S = DanaMaster(N, W, MODE_SA, Hyper(eta, gamma, f32=False), np.float64)
    S.run_buffers((np.arange(400) % W).astype(np.uint32), c[None, :])
    assert np.allclose(S.vw, np.tile(c / W / (1 - gamma), (W, 1)), rtol=1e-10)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_dana_ga_dyadic_one_step(dtype):
    # Alg. 8 + Alg. 14 on exact binary numbers (same Gap numbers as the momentum example):
    # C = 1/8, Graw = 4, G = 5 -> g/G = 2; v^i: 1/4 -> 1/2*1/4 + 2 = 2.125; theta = 1 - 1/4*2.125 = 0.46875;
    # sum: 1 -> (1 - 1/4) + 2.125 = 2.875; eta*gamma = 1/8 -> look-ahead 0.46875 - 0.359375 = 0.109375; m = 2.2734375.
    h = Hyper(eta=0.5, gamma=0.5, beta=0.5, eps=0.0, eta_k=0.25, f32=False)
    th, vi, vs = np.array([1.0], dtype), np.array([0.25], dtype), np.array([1.0], dtype)
    m, s, g = np.array([0.03125], dtype), np.array([0.5], dtype), np.array([10.0], dtype)
    sfx = "f32" if dtype == np.float32 else "f64"
    getattr(oracle.lib(), "orc_dana_step_" + sfx)(1, *(x.ctypes.data for x in (th, vi, vs, m, s, g)), MODE_GA, 2, 3,
                                                  *h.args(), 0)
    assert (vi[0], th[0], vs[0], s[0], m[0]) == (2.125, 0.46875, 2.875, 0.109375, 2.2734375)


# ------------------------------------------------------------------ Adam
def test_adam_single_worker_matches_torch_adam():
    N, T, lr = 40, 200, 0.01
    a, ts = quad_inputs(N, 4, np.float64)
    A = AdamMaster(N, 1, MODE_ASGD, Hyper(lr, 0.0, f32=False), np.float64, beta1=0.9, beta2=0.999, adam_eps=1e-8)
    A.run_quadratic(np.zeros(T, np.uint32), a, ts, seed=0, sigma=0.0)
    p = torch.zeros(N, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=lr, betas=(0.9, 0.999), eps=1e-8)
    ta, tts = torch.from_numpy(a), torch.from_numpy(ts)
    for _ in range(T):
        opt.zero_grad()
        (0.5 * (ta * (p - tts) ** 2).sum()).backward()
        opt.step()
    assert np.allclose(A.theta, p.detach().numpy(), rtol=1e-9, atol=1e-12)
    assert np.linalg.norm(A.theta) > 0.1


def test_adam_single_worker_all_penalties_bit_identical():
    N, T = 300, 50
    a, ts = quad_inputs(N, 6, np.float32)
    ref = None
    for mode in PENALTIES:
        A = AdamMaster(N, 1, mode, Hyper(0.01, 0.0), np.float32)
        A.run_quadratic(np.zeros(T, np.uint32), a, ts, seed=3)
        ref = A.theta.copy() if ref is None else ref
        assert np.array_equal(A.theta, ref), mode


@pytest.mark.parametrize("mode,div", [(MODE_SA, lambda W: W), (MODE_GA, lambda W: W), (MODE_GA_HINGE, lambda W: W - 1)])
def test_adam_penalised_steady_state_step(mode, div):
    # round robin over W workers, the same gradient c: v2-hat = c^2 at every step (bias corrected),
    # m1-hat -> c / G, so the update vector settles at sign(c)/G with G = tau = W (SA, Alg. 10), and for
    # the Gap (Alg. 11): C -> eta |u|, a snapshot W-1 steps old gives Graw = W-1, G = W (hinge: W-1).
    N, W, T, lr = 3, 5, 1500, 0.01
    c = np.array([2.0, -0.5, 7.0])
    A = AdamMaster(N, W, mode, Hyper(lr, 0.0, beta=0.9, eps=1e-12, f32=False), np.float64, beta1=0.9, beta2=0.999,
                   adam_eps=1e-12)
    sched = (np.arange(T) % W).astype(np.uint32)
    A.run_buffers(sched[:-1], c[None, :])
    before = A.theta.copy()
    A.apply(int(sched[-1]), c)
    assert np.allclose(before - A.theta, lr * np.sign(c) / div(W), rtol=1e-6)
    # the second moment never sees the penalty (App. C.1): v2 = (1 - beta2^K) c^2
    assert np.allclose(A.v2, (1 - 0.999 ** T) * c ** 2, rtol=1e-12)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_adam_ga_dyadic_one_step(dtype):
    # beta1 = beta2 = 0, adam eps = 0, hinge Gap with C = 1/8, Graw = 4 -> G = 4:
    # coefficient (1 - 0)/4 = 1/4; m1 = 2.5; v2 = 100; u = 2.5/10 = 1/4; theta = 1 - 1/4*1/4 = 0.9375;
    # c = 1/2 * 1/32 + 1/2 * 1/16 = 0.046875.
    h = Hyper(eta=0.5, gamma=0.0, beta=0.5, eps=0.0, eta_k=0.25, f32=False)
    th, m1, v2 = np.array([1.0], dtype), np.array([9.0], dtype), np.array([9.0], dtype)
    c, s, g = np.array([0.03125], dtype), np.array([0.5], dtype), np.array([10.0], dtype)
    sfx = "f32" if dtype == np.float32 else "f64"
    getattr(oracle.lib(), "orc_adam_step_" + sfx)(1, *(x.ctypes.data for x in (th, m1, v2, c, s, g)), MODE_GA_HINGE, 2,
                                                  3, h.eta_k, h.eta_max, h.beta, h.eps, 0.0, 0.0, 0.0, 0)
    assert (m1[0], v2[0], th[0], c[0], s[0]) == (2.5, 100.0, 0.9375, 0.046875, 0.9375)


def test_families_reach_the_minimum():
    N, W, T = 3, 4, 6000
    a, ts = quad_inputs(N, 8, np.float64)
    sched = oracle.simulate_schedule(W, T, seed=2)
    for mode in (MODE_SA, MODE_GA):
        D = DanaMaster(N, W, mode, Hyper(0.1, 0.9, f32=False), np.float64)
        D.run_quadratic(sched, a, ts, seed=0, sigma=0.0)
        assert np.abs(D.theta - ts).max() < 0.01 * np.abs(ts).max(), mode
        A = AdamMaster(N, W, mode, Hyper(0.01, 0.0, f32=False), np.float64)
        A.run_quadratic(sched, a, ts, seed=0, sigma=0.0)
        assert np.abs(A.theta - ts).max() < 0.02 * np.abs(ts).max(), mode


# ------------------------------------------------------------------ layer-wise and global Gap
from oracle import LayerwiseMaster


@pytest.mark.parametrize("mode", [MODE_GA, MODE_GA_HINGE])
def test_layers_of_one_parameter_are_the_parameter_wise_gap(mode):
    # Eq. 4 with every layer a single parameter is Eq. 5: ||x|| = |x| and the summed m-hat is m-hat itself.
    N, W, T = 300, 4, 150
    a, ts = quad_inputs(N, 5, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=5)
    L = LayerwiseMaster(N, W, mode, Hyper(), np.ones(N, np.uint64), np.float32)
    M = Master(N, W, mode, Hyper(), np.float32)
    L.run_quadratic(sched, a, ts, seed=9)
    M.run_quadratic(sched, a, ts, seed=9)
    assert np.array_equal(L.theta, M.theta) and np.array_equal(L.m, M.m) and np.array_equal(L.snaps, M.snaps)


@pytest.mark.parametrize("layers", [[40], [1, 7, 32], [13, 27]])
def test_layer_gap_constant_gradient_equals_delay(layers):
    # ASGD-like history (gamma = 0, huge eta_max so that the penalty is ~1 while m is built), then read the Gap:
    # build the state with the plain master, then one layer-wise step.  Every update was -eta c, so a snapshot
    # s steps old has ||theta - theta^i|| = s eta ||c||, C_p = eta (||c_p|| + eps): G_p = s + 1 for every layer,
    # whatever its size (remark after Def. 1).
    N, W, eta = 40, 4, 0.1
    c = np.linspace(0.5, 3.0, N) * np.where(np.arange(N) % 3, 1, -1)
    P = Master(N, W, MODE_ASGD, Hyper(eta, 0.0, f32=False), np.float64, track_gap=True)
    sched = np.array([0, 1, 2, 3, 0, 1, 2, 0, 1, 0, 0], np.uint32)
    P.run_buffers(sched, c[None, :])
    L = LayerwiseMaster(N, W, MODE_GA, Hyper(eta, 0.0, f32=False), layers, np.float64)
    L.theta[:], L.v[:], L.m[:], L.snaps[:], L.k, L.iter[:] = P.theta, P.v, P.m, P.snaps, P.k, P.iter
    age = P.k - int(P.iter[3])                      # worker 3 was last seen `age` steps ago
    th_before = L.theta.copy()
    L.apply(3, c)
    assert np.allclose(L.last_gaps, age + 1, rtol=1e-7)
    assert np.allclose(th_before - L.theta, eta * c / (age + 1), rtol=1e-7)      # one penalty for the whole layer


def test_global_gap_is_scale_free_and_uniform():
    N, W, T = 200, 4, 80
    a, ts = quad_inputs(N, 3, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=3)
    out = []
    for s in (1.0, 256.0):
        L = LayerwiseMaster(N, W, MODE_GA, Hyper(eps=float(np.float32(1e-8)) * s), None, np.float32)
        L.run_quadratic(sched, a, ts * np.float32(s), seed=4, sigma=float(np.float32(0.01)) * s)
        out.append(L.theta / np.float32(s))
    assert np.array_equal(out[0], out[1])
    # the penalty is one number per layer: v' - gamma v is g / G with the same G for every parameter
    L = LayerwiseMaster(N, W, MODE_GA, Hyper(f32=False), [50, 150], np.float64)
    L.run_quadratic(sched, a.astype(np.float64), ts.astype(np.float64), seed=4)
    v0 = L.v.copy()
    w = int(sched[0])
    g = oracle.quadratic_gradient(L.snaps[w], a.astype(np.float64), ts.astype(np.float64), 4, L.k + 1, 0.01)
    L.apply(w, g)
    ratio = g / (L.v - 0.9 * v0)
    assert np.allclose(ratio[:50], L.last_gaps[0], rtol=1e-9) and np.allclose(ratio[50:], L.last_gaps[1], rtol=1e-9)
    assert abs(L.last_gaps[0] - L.last_gaps[1]) > 1e-6


# ------------------------------------------------------------------ Nesterov form
def test_nesterov_single_worker_matches_torch_sgd():
    N, T, lr, gamma = 30, 150, 0.05, 0.9
    a, ts = quad_inputs(N, 11, np.float64)
    M = Master(N, 1, MODE_GA, Hyper(lr, gamma, f32=False), np.float64, nesterov=True)
    M.run_quadratic(np.zeros(T, np.uint32), a, ts, seed=0, sigma=0.0)
    p = torch.zeros(N, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=lr, momentum=gamma, nesterov=True)
    ta, tts = torch.from_numpy(a), torch.from_numpy(ts)
    for _ in range(T):
        opt.zero_grad()
        (0.5 * (ta * (p - tts) ** 2).sum()).backward()
        opt.step()
    assert np.allclose(M.theta, p.detach().numpy(), rtol=1e-11, atol=1e-13)
    H = Master(N, 1, MODE_GA, Hyper(lr, gamma, f32=False), np.float64)
    H.run_quadratic(np.zeros(T, np.uint32), a, ts, seed=0, sigma=0.0)
    assert not np.allclose(H.theta, M.theta, rtol=1e-4)              # it is not the heavy-ball trajectory


@pytest.mark.parametrize("mode", [MODE_ASGD, MODE_SA, MODE_GA, MODE_GA_HINGE])
def test_nesterov_without_momentum_is_plain(mode):
    N, W, T = 200, 4, 80
    a, ts = quad_inputs(N, 13, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=13)
    A = Master(N, W, mode, Hyper(0.1, 0.0), np.float32, nesterov=True)
    B = Master(N, W, mode, Hyper(0.1, 0.0), np.float32)
    A.run_quadratic(sched, a, ts, seed=1)
    B.run_quadratic(sched, a, ts, seed=1)
    assert np.array_equal(A.theta, B.theta) and np.array_equal(A.snaps, B.snaps)


def test_nesterov_gap_penalty_fixed_point():
    # same construction as for the heavy-ball master, gamma = 0.5: with every penalised gradient equal to
    # c/G the update vector settles at d = (c/G)(1 + gamma/(1-gamma)); C follows d, so Graw = W-1 and G = W.
    N, W, T, eta, gamma = 3, 5, 2500, 0.05, 0.5
    c = np.array([0.4, -1.5, 3.0])
    M = Master(N, W, MODE_GA, Hyper(eta, gamma, beta=0.9, eps=1e-12, f32=False), np.float64, nesterov=True)
    M.run_buffers((np.arange(T) % W).astype(np.uint32), np.ascontiguousarray(c[None, :]))
    assert np.allclose(M.v, (c / W) / (1 - gamma), rtol=1e-6)
