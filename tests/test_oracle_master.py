"""Pins for the oracle's master update (no GPU).

Each test checks the oracle against something the paper or the mathematics
fixes, not against a second copy of its own loop:
  * heavy-ball momentum (Sec. 2)                       -> matrix-power closed form
  * no Gap without intervening updates (Sec. 4.1)      -> W = 1 makes all modes equal
  * SA-gradient divides g by tau (Alg. 5)              -> harmonic-sum closed form
  * SA step-size form, two-step expansion (Sec. 3.1)   -> the printed identity
  * C coefficient (Alg. 14) and Gap = delay when all updates point the same
    way (remark after Def. 1)                          -> constant-gradient closed form
  * Gap penalty 1/G on the gradient (Alg. 4)           -> dyadic one-step example, fixed point
  * Gap is scale free (Def. 1: C is a distance)        -> power-of-two rescaling is bit exact
  * parameter-wise independence (Sec. 4.3)             -> subset runs equal the full run
"""
import numpy as np
import pytest

import ga_inputs
import oracle
from oracle import MODE_ASGD, MODE_GA, MODE_GA_HINGE, MODE_SA, MODE_SA_STEP, Hyper, Master

ALL_MODES = [MODE_ASGD, MODE_SA, MODE_SA_STEP, MODE_GA, MODE_GA_HINGE]


def quad_inputs(N, seed, dtype):
    return ga_inputs.curvatures(N, seed).astype(dtype), ga_inputs.optimum(N, seed).astype(dtype)


# ---------------------------------------------------------------- momentum
@pytest.mark.parametrize("gamma", [0.9, 0.0, -0.5])
def test_single_worker_matches_heavy_ball_closed_form(gamma):
    # noise-free quadratic, one worker: g_k = a (theta_k - theta*), so per coordinate
    # [e; v]_{k+1} = A [e; v]_k with e = theta - theta*, A = [[1 - eta a, -eta gamma], [a, gamma]].
    N, T, eta = 64, 200, 0.1
    a, ts = quad_inputs(N, 3, np.float64)
    sched = np.zeros(T, dtype=np.uint32)
    expect = np.empty(N)
    for j in range(N):
        A = np.array([[1 - eta * a[j], -eta * gamma], [a[j], gamma]])
        e = np.linalg.matrix_power(A, T) @ np.array([0.0 - ts[j], 0.0])
        expect[j] = ts[j] + e[0]
    for mode in ALL_MODES:
        M = Master(N, 1, mode, Hyper(eta, gamma, f32=False), np.float64)
        M.run_quadratic(sched, a, ts, seed=0, sigma=0.0)
        assert np.allclose(M.theta, expect, rtol=1e-10, atol=1e-12), mode
    M32 = Master(N, 1, MODE_GA, Hyper(eta, gamma), np.float32)
    M32.run_quadratic(sched, a.astype(np.float32), ts.astype(np.float32), seed=0, sigma=0.0)
    assert np.allclose(M32.theta, expect, rtol=2e-4, atol=2e-5)


def test_single_worker_all_modes_bit_identical():
    # With one worker the master's parameters never move between send and
    # receive: the Gap term is zero, tau = 1, and every penalty is exactly 1.
    N, T = 1000, 60
    a, ts = quad_inputs(N, 5, np.float32)
    sched = np.zeros(T, dtype=np.uint32)
    ref = None
    for mode in ALL_MODES:
        M = Master(N, 1, mode, Hyper(), np.float32)
        tau = M.run_quadratic(sched, a, ts, seed=17, sigma=0.01)
        assert np.all(tau == 1)
        if ref is None:
            ref = (M.theta.copy(), M.v.copy())
        assert np.array_equal(M.theta, ref[0]) and np.array_equal(M.v, ref[1]), mode
        assert np.array_equal(M.snaps[0], M.theta)


def test_plain_sgd_sum_when_gamma_zero():
    # Alg. 2 with gamma = 0: theta_K = theta_0 - eta * sum of the gradients received.
    N, W, T = 50, 4, 40
    rng = np.random.default_rng(0)
    bufs = rng.standard_normal((W, N))
    sched = rng.integers(0, W, T).astype(np.uint32)
    M = Master(N, W, MODE_ASGD, Hyper(0.05, 0.0, f32=False), np.float64, theta0=rng.standard_normal(N))
    th0 = M.theta.copy()
    M.run_buffers(sched, bufs, pick_by_worker=True)
    assert np.allclose(M.theta, th0 - 0.05 * bufs[sched].sum(0), rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- SA
def test_sa_gradient_harmonic_closed_form():
    # Alg. 5, gamma = 0, the same gradient c from everyone, round robin over W:
    # tau_k = min(k, W), theta_K = -eta c sum_k 1/tau_k.
    N, W, T, eta = 8, 6, 30, 0.1
    c = np.linspace(-2, 2, N)
    bufs = np.tile(c, (1, 1))
    sched = (np.arange(T) % W).astype(np.uint32)
    M = Master(N, W, MODE_SA, Hyper(eta, 0.0, f32=False), np.float64)
    tau = M.run_buffers(sched, bufs)
    assert tau.tolist() == [min(k, W) for k in range(1, T + 1)]
    H = sum(1.0 / min(k, W) for k in range(1, T + 1))
    assert np.allclose(M.theta, -eta * c * H, rtol=1e-13, atol=0)
    # step-size form (Alg. 3) coincides with the gradient form when gamma = 0
    M2 = Master(N, W, MODE_SA_STEP, Hyper(eta, 0.0, f32=False), np.float64)
    M2.run_buffers(sched, bufs)
    assert np.allclose(M2.theta, M.theta, rtol=1e-13, atol=0)
    # and differs once there is momentum (the under-penalisation of Sec. 3.1)
    Ma = Master(N, W, MODE_SA, Hyper(eta, 0.9, f32=False), np.float64)
    Mb = Master(N, W, MODE_SA_STEP, Hyper(eta, 0.9, f32=False), np.float64)
    Ma.run_buffers(sched, bufs)
    Mb.run_buffers(sched, bufs)
    assert not np.allclose(Ma.theta, Mb.theta, rtol=1e-3)


def test_sa_step_two_step_identity():
    # Sec. 3.1: theta_{k+2} = theta_{k+1} - (eta/tau_{k+1}) (gamma^2 v_k + gamma g_k + g_{k+1}).
    N, W, eta, gamma = 16, 3, 0.1, 0.9
    rng = np.random.default_rng(1)
    M = Master(N, W, MODE_SA_STEP, Hyper(eta, gamma, f32=False), np.float64, theta0=rng.standard_normal(N))
    M.v[:] = rng.standard_normal(N)
    # put the master at step 7 with worker 2 last seen at 1 (tau = 7) and worker 0 at 7... (tau = 2 next)
    M.k = 7
    M.iter[:] = [7, 5, 1]
    v_k, th_k = M.v.copy(), M.theta.copy()
    g_k, g_k1 = rng.standard_normal(N), rng.standard_normal(N)
    assert M.apply(2, g_k) == 7                    # stale gradient
    th_k1 = M.theta.copy()
    assert np.allclose(th_k1, th_k - (eta / 7) * (gamma * v_k + g_k), rtol=1e-13)
    assert M.apply(0, g_k1) == 2                   # fast worker
    expect = th_k1 - (eta / 2) * (gamma ** 2 * v_k + gamma * g_k + g_k1)
    assert np.allclose(M.theta, expect, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- C coefficient and the Gap
@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-7), (np.float32, 2e-5)])
def test_constant_gradient_gap_equals_delay(dtype, tol):
    # ASGD, gamma = 0, every worker sends the same c: v = c at every step, so
    # m_k = (1 - beta^k) c^2, m-hat = c^2 and C = eta_max (|c| + eps) for every k (Alg. 14).
    # A worker whose snapshot is s master steps old sees |theta - theta^i| = s eta |c|,
    # i.e. Graw = s and the paper's Gap = s + 1 = its delay at the next arrival:
    # "E[G_k] = tau_k only if all previous updates were in the exact same direction".
    N, W, T, eta = 32, 5, 57, 0.1
    c = np.linspace(0.5, 3.0, N).astype(dtype) * np.where(np.arange(N) % 2, 1, -1).astype(dtype)
    bufs = np.ascontiguousarray(c[None, :])
    rng = np.random.default_rng(2)
    sched = rng.integers(0, W, T).astype(np.uint32)
    sched[-W:] = rng.permutation(W)                 # everyone has arrived at least once
    M = Master(N, W, MODE_ASGD, Hyper(eta, 0.0, f32=(dtype == np.float32)), dtype, track_gap=True)
    M.run_buffers(sched, bufs)
    assert np.allclose(M.m, (1 - 0.999 ** T) * c.astype(np.float64) ** 2, rtol=50 * tol)
    for w in range(W):
        age = M.k - int(M.iter[w])                   # master steps since w's snapshot
        st = M.gap_statistics(w)
        assert abs(st["mean_graw"] - age) <= tol * max(1, age), (w, age, st)
        assert st["frac_gt0"] == (1.0 if age > 0 else 0.0)
        assert st["n_nonfinite"] == 0
    # changing eta_k later must not change C: it is tied to eta_max
    w = int(np.argmax(M.k - M.iter.astype(np.int64)))
    before = M.gap_statistics(w)["mean_graw"]
    M.hyper.eta_k = M.hyper.eta_k / 4
    assert M.gap_statistics(w)["mean_graw"] == before
    M.hyper.eta_max = M.hyper.eta_max / 4
    assert abs(M.gap_statistics(w)["mean_graw"] - 4 * before) < 1e-4 * before


def test_first_step_coefficient():
    # After the first arrival the bias correction cancels: m-hat_1 = v_2^2, C_1 = eta_max (|v_2| + eps).
    # Second arrival from another worker (snapshot still theta_0): |theta - theta^i| = eta |v_2|,
    # so Graw = |v_2| / (|v_2| + eps) ~ 1, paper's penalty ~ 1/2, hinge penalty exactly 1.
    N, eta = 40, 0.1
    rng = np.random.default_rng(3)
    g1, g2 = rng.standard_normal(N), rng.standard_normal(N)
    for mode, pen in [(MODE_GA, 0.5), (MODE_GA_HINGE, 1.0)]:
        M = Master(N, 2, mode, Hyper(eta, 0.9, f32=False), np.float64)
        M.apply(0, g1)
        assert np.allclose(M.v, g1, rtol=0, atol=0)                 # Gap is zero at k = 1
        assert np.allclose(M.m, 0.001 * g1 ** 2, rtol=1e-12)
        st = M.gap_statistics(1)
        assert abs(st["mean_graw"] - 1.0) < 1e-6
        M.apply(1, g2)
        assert np.allclose(M.v, 0.9 * g1 + pen * g2, rtol=1e-6, atol=1e-9), mode


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_dyadic_one_step_example(dtype):
    # Alg. 4 + Alg. 14 on numbers that are exact in binary, worked by hand:
    # beta = 1/2, k = 2: 1/(1 - beta^(k-1)) = 2.  m_1 = 1/32 -> m-hat = 1/16 -> sqrt = 1/4;
    # eps = 0, eta_max = 1/2 -> C = 1/8.  theta = 1, theta^i = 1/2 -> |diff| = 1/2 -> Graw = 4.
    # Paper: G = 5, g = 10 -> g/G = 2;  v' = 1/2 * 1/4 + 2 = 2.125;  eta_k = 1/4 -> theta' = 1 - 0.53125.
    # m' = 1/2 * 1/32 + 1/2 * 2.125^2 = 2.2734375.
    # Hinge: G = 4 -> g/G = 2.5; v' = 2.625; theta' = 1 - 0.65625; m' = 1/64 + 3.4453125.
    h = Hyper(eta=0.5, gamma=0.5, beta=0.5, eps=0.0, eta_k=0.25, f32=False)
    for mode, v1, th1, m1 in [(MODE_GA, 2.125, 0.46875, 2.2734375), (MODE_GA_HINGE, 2.625, 0.34375, 3.4609375)]:
        th, v, m = np.array([1.0], dtype), np.array([0.25], dtype), np.array([0.03125], dtype)
        s, g = np.array([0.5], dtype), np.array([10.0], dtype)
        oracle.step(th, v, m, s, g, mode, k=2, tau=3, hyper=h)
        assert (v[0], th[0], m[0], s[0]) == (v1, th1, m1, th1)
    # negative difference and negative gradient: the Gap uses |diff|, the sign of g survives
    th, v, m = np.array([0.5], dtype), np.array([0.25], dtype), np.array([0.03125], dtype)
    s, g = np.array([1.0], dtype), np.array([-10.0], dtype)
    oracle.step(th, v, m, s, g, MODE_GA, k=2, tau=3, hyper=h)
    assert (v[0], th[0]) == (-1.875, 0.5 + 0.46875)
    # SA on the same numbers: g / tau (Alg. 5) and eta / tau (Alg. 3), tau = 4
    th, v, m = np.array([1.0], dtype), np.array([0.25], dtype), np.array([0.0], dtype)
    s = np.array([0.5], dtype)
    oracle.step(th, v, m, s, np.array([10.0], dtype), MODE_SA, k=9, tau=4, hyper=h)
    assert (v[0], th[0], m[0]) == (2.625, 1 - 0.65625, 0.0)         # m untouched without tracking
    th, v = np.array([1.0], dtype), np.array([0.25], dtype)
    oracle.step(th, v, m, s, np.array([10.0], dtype), MODE_SA_STEP, k=9, tau=4, hyper=h)
    assert (v[0], th[0]) == (10.125, 1 - 0.0625 * 10.125)


@pytest.mark.parametrize("mode,limit", [(MODE_GA, lambda W: W), (MODE_GA_HINGE, lambda W: W - 1)])
def test_gap_penalty_fixed_point_equals_delay(mode, limit):
    # GA, gamma = 0, same gradient c from everyone, round robin over W workers.
    # If every step has size c/p then C -> eta |c|/p and a snapshot W-1 steps old gives
    # Graw = W-1, so p = W (paper: Graw + 1) or W-1 (hinge): the penalty settles at
    # the delay tau = W, the bound the paper states for aligned updates (after Def. 1).
    N, W, T, eta = 4, 6, 1500, 0.1
    c = np.array([0.3, -1.0, 2.0, 5.0])
    M = Master(N, W, mode, Hyper(eta, 0.0, beta=0.9, eps=1e-12, f32=False), np.float64)
    M.run_buffers((np.arange(T) % W).astype(np.uint32), np.ascontiguousarray(c[None, :]))
    assert np.allclose(M.v, c / limit(W), rtol=1e-6)


@pytest.mark.parametrize("mode", [MODE_GA, MODE_GA_HINGE])
def test_gap_is_scale_free(mode):
    # Def. 1 measures distance in units of C, itself a distance: scaling the problem
    # (theta*, noise, and the guard eps that is added to a distance) by a power of two
    # scales the whole trajectory by it, bit for bit.
    N, W, T = 500, 4, 300
    a, ts = quad_inputs(N, 9, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=9)
    out = []
    for s in (1.0, 1024.0):
        M = Master(N, W, mode, Hyper(eps=float(np.float32(1e-8)) * s), np.float32)
        M.run_quadratic(sched, a, (ts * np.float32(s)), seed=4, sigma=float(np.float32(0.01)) * s)
        out.append(M.theta / np.float32(s))
    assert np.array_equal(out[0], out[1])
    assert np.linalg.norm(out[0]) > 0


@pytest.mark.parametrize("mode", [MODE_GA, MODE_GA_HINGE])
def test_gap_zero_means_no_penalty_and_large_gap_divides(mode):
    N = 1000
    th, v, m, snaps = ga_inputs.random_state(N, 1, 6)
    g = ga_inputs.rng(6, 9).standard_normal(N, dtype=np.float32)
    h = Hyper()
    # snapshot equal to theta: identical to the momentum step of Alg. 2
    a = [x.copy() for x in (th, v, m)]
    b = [x.copy() for x in (th, v, m)]
    sa, sb = th.copy(), th.copy()
    oracle.step(*a, sa, g, mode, 50, 7, h)
    oracle.step(*b, sb, g, MODE_ASGD, 50, 7, h, track_gap=True)
    for x, y in zip(a + [sa], b + [sb]):
        assert np.array_equal(x, y)
    # generic snapshot: v' - gamma v must equal g / G with G rebuilt in double from the
    # state (|diff|, m, 1 - beta^(k-1)); checks the 1/G placement and the bias correction
    t2, v2, m2, s2 = th.copy(), v.copy(), m.copy(), snaps[0].copy()
    oracle.step(t2, v2, m2, s2, g, mode, 50, 7, h)
    bc = 1 - np.float64(h.beta) ** 49
    C = h.eta_max * (np.sqrt(m.astype(np.float64) / bc) + h.eps)
    graw = np.abs(th.astype(np.float64) - snaps[0]) / C
    G = 1 + graw if mode == MODE_GA else np.maximum(1, graw)
    got = v2.astype(np.float64) - np.float64(h.gamma) * v
    assert np.allclose(got, g / G, rtol=2e-5, atol=2e-7)
    assert np.array_equal(s2, t2)


# ---------------------------------------------------------------- structure
def test_snapshots_and_bookkeeping():
    N, W, T = 64, 5, 200
    a, ts = quad_inputs(N, 2, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=8)
    M = Master(N, W, MODE_GA, Hyper(), np.float32)
    hist = {}
    for k, w in enumerate(sched, start=1):
        w = int(w)
        others = {u: M.snaps[u].copy() for u in range(W) if u != w}
        g = oracle.quadratic_gradient(M.snaps[w], a, ts, seed=1, k=k)
        M.apply(w, g)
        assert np.array_equal(M.snaps[w], M.theta)           # save and send theta_{k+1}
        for u, s in others.items():
            assert np.array_equal(M.snaps[u], s)
        hist[w] = M.theta.copy()
    tau, it = oracle.delays(W, sched)
    assert M.tau_log == tau.tolist() and np.array_equal(M.iter, it) and M.k == T
    for w, s in hist.items():
        assert np.array_equal(M.snaps[w], s)
    # the fused loop (run_quadratic) is the same trajectory as apply-by-apply
    M2 = Master(N, W, MODE_GA, Hyper(), np.float32)
    M2.run_quadratic(sched, a, ts, seed=1)
    assert np.array_equal(M2.theta, M.theta) and np.array_equal(M2.snaps, M.snaps)


def test_parameter_wise_independence():
    # Sec. 4.3: every parameter is penalised independently, so a gathered subset
    # (with its global indices for the noise) reproduces the full run exactly.
    N, W, T = 3001, 6, 120
    a, ts = quad_inputs(N, 12, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=3)
    for mode in (MODE_GA, MODE_SA):
        full = Master(N, W, mode, Hyper(), np.float32)
        full.run_quadratic(sched, a, ts, seed=77)
        idx = ga_inputs.sample_indices(N, 100, 1)[::7].copy()
        sub = Master(idx.size, W, mode, Hyper(), np.float32)
        sub.run_quadratic(sched, a[idx], ts[idx], seed=77, idx=idx)
        assert np.array_equal(sub.theta, full.theta[idx])
        assert np.array_equal(sub.snaps, full.snaps[:, idx])
        assert np.array_equal(sub.m, full.m[idx])


def test_quadratic_gradient_is_the_gradient():
    # g(sigma = 0) is the gradient of f(theta) = 1/2 sum a (theta - theta*)^2: central differences.
    N = 12
    a, ts = quad_inputs(N, 4, np.float64)
    x = np.random.default_rng(0).standard_normal(N)
    f = lambda y: 0.5 * np.sum(a * (y - ts) ** 2)
    g = oracle.quadratic_gradient(x, a, ts, seed=0, k=1, sigma=0.0)
    for j in range(N):
        e = np.zeros(N)
        e[j] = 1e-6
        assert abs((f(x + e) - f(x - e)) / 2e-6 - g[j]) < 1e-8
    # the noise term is sigma * z(seed, k, j), added as is
    g2 = oracle.quadratic_gradient(x, a, ts, seed=5, k=3, sigma=0.01)
    assert np.allclose(g2 - g, 0.01 * oracle.noise_f32(5, 3, 0, N).astype(np.float64), rtol=0, atol=1e-12)


def delayed_gradient_descent(schedule, W, a, ts, eta, divide_by_tau):
    """theta_{k+1} = theta_k - eta_k grad f(theta_{k - tau_k}) (Sec. 2, the ASGD rule without momentum) written on
    the whole history of iterates: the arriving worker's gradient is taken at the iterate that existed right after
    its previous arrival (iterate 0 before its first).  SA: eta_k = eta / tau_k (Alg. 3 / Alg. 5 coincide for
    gamma = 0)."""
    hist = [np.zeros_like(ts)]
    last = [0] * W
    for k, w in enumerate(schedule, start=1):
        tau = k - last[w]
        stale = hist[k - tau]
        lr = eta / tau if divide_by_tau else eta
        hist.append(hist[-1] - lr * (a * (stale - ts)))
        last[w] = k
    return np.array(hist)


@pytest.mark.parametrize("schedule_kind", ["round_robin", "simulated"])
def test_without_momentum_the_master_is_delayed_gradient_descent(schedule_kind):
    # gamma = 0, no noise: the snapshot mechanism of Alg. 2 / Alg. 5 ("save and send", theta^i) must reproduce
    # the textbook recursion on stale iterates, step by step.  Round robin: tau_k = min(k, W) in closed form.
    N, W, T, eta = 5, 4, 300, 0.1
    a, ts = quad_inputs(N, 8, np.float64)
    sched = (np.arange(T) % W).astype(np.uint32) if schedule_kind == "round_robin" else oracle.simulate_schedule(W, T, seed=4)
    for mode, div in ((MODE_ASGD, False), (MODE_SA, True), (MODE_SA_STEP, True)):
        ref = delayed_gradient_descent([int(w) for w in sched], W, a, ts, eta, div)
        M = Master(N, W, mode, Hyper(eta, 0.0, f32=False), np.float64)
        for k in range(T):
            M.run_quadratic(sched[k:k + 1], a, ts, seed=0, sigma=0.0)
            assert np.allclose(M.theta, ref[k + 1], rtol=1e-12, atol=1e-15), (mode, k)
        if schedule_kind == "round_robin":
            assert M.tau_log == [min(k, W) for k in range(1, T + 1)]


def test_minimum_of_the_quadratic_is_reached():
    # Brute force on a tiny problem: the grid minimiser of f is theta*.  Then, without momentum and without
    # noise, every penalised master is x_{k+1} = x_k - c_k x_{k-d_k} for the error x = theta - theta*, with
    # 0 < c_k <= c = eta max(a) (every penalty divides by a number >= 1) and d_k = tau_k - 1.  If the error keeps
    # its sign and shrinks per step by no more than a factor rho, then x_{k-d} <= x_k rho^-d, and the step is
    # self-consistent when c_k rho^-d_k <= 1 - rho: the error never changes sign and never grows.
    #   * round robin over W = 3 workers (d = 2), any penalty: c rho^-2 <= 1 - rho holds for rho = 0.9, c <= 0.081;
    #   * simulated schedule, SA: c_k = c / tau_k, and (c / tau) rho^-(tau - 1) <= 1 - rho for every delay that occurs.
    # For SA the contraction is bounded as well: the stale error is at least the current one, so step k shrinks
    # the error at least by the factor 1 - eta a / tau_k.
    N, W, T, eta = 3, 3, 4000, 0.1
    a, ts = quad_inputs(N, 8, np.float64)
    grid = np.linspace(-4, 4, 161)
    for j in range(N):
        assert abs(grid[np.argmin(0.5 * a[j] * (grid - ts[j]) ** 2)] - ts[j]) <= 0.025 + 1e-12
    c, rho = eta * a.max(), 0.9
    assert c * rho ** -2 <= 1 - rho
    simulated = oracle.simulate_schedule(W, T, seed=2)
    taus = oracle.delays(W, simulated)[0].astype(np.float64)
    assert np.all(c / taus * rho ** -(taus - 1) <= 1 - rho)
    round_robin = (np.arange(T) % W).astype(np.uint32)
    for mode, sched in ((MODE_SA, simulated), (MODE_SA, round_robin), (MODE_GA, round_robin), (MODE_GA_HINGE, round_robin)):
        M = Master(N, W, mode, Hyper(eta, 0.0, f32=False), np.float64)
        err = [-ts.copy()]
        for k in range(T):
            M.run_quadratic(sched[k:k + 1], a, ts, seed=0, sigma=0.0)
            err.append(M.theta - ts)
        err = np.array(err)
        live = np.abs(err[1:]) > 1e-12                                           # above the rounding floor of the run
        assert np.all((np.sign(err[1:]) == np.sign(err[0])) | ~live), mode       # no overshoot
        assert np.all((np.abs(err[1:]) <= np.abs(err[:-1])) | ~live), mode       # monotone
        if mode == MODE_SA:
            rate = np.prod(1.0 - eta * a[None, :] / np.array(M.tau_log)[:, None], axis=0)
            assert np.all(np.abs(err[-1]) <= rate * np.abs(err[0]) + 1e-12)
            assert np.abs(err[-1]).max() < 1e-6 * np.abs(ts).max()
        else:
            assert np.abs(err[-1]).max() < np.abs(err[0]).max()                  # descends; how fast is not fixed


# ---------------------------------------------------------------- which vector feeds Alg. 14
def gap_aware_in_numpy(sched, W, a, ts, eta, gamma, beta, eps, raw_input):
    """Alg. 4 with Alg. 14 in plain numpy (double).  raw_input: Alg. 14 exactly as printed, with a momentum
    buffer of its own fed by the raw gradient; otherwise the reading taken here, fed by the update vector."""
    N = a.size
    theta, v, u, m = np.zeros(N), np.zeros(N), np.zeros(N), np.zeros(N)
    snaps = np.zeros((W, N))
    c_sum = np.zeros(N)
    for k, w in enumerate(sched, start=1):
        g = a * (snaps[w] - ts)
        mhat = m / (1.0 - beta ** (k - 1)) if k > 1 else np.zeros(N)
        C = eta * (np.sqrt(mhat) + eps)
        c_sum += C
        G = np.abs(theta - snaps[w]) / C + 1.0
        v = gamma * v + g / G
        theta = theta - eta * v
        u = gamma * u + g
        fed = u if raw_input else v
        m = beta * m + (1.0 - beta) * fed * fed
        snaps[w] = theta
    return theta, c_sum / len(sched)


def test_reading_of_the_input_of_alg14_is_recorded():
    # Alg. 14 prints v <- gamma v + g with the raw gradient; Alg. 4's v holds g / G.  This library keeps one v (the
    # update vector) and feeds Alg. 14 with it.  The paper does not fix that choice, so nothing pins it: this test
    # records what it changes.  (1) With one worker there is no Gap, G = 1, and both forms are the same numbers.
    # (2) With eight workers the reading gives a smaller C (its input is the penalised vector), hence larger
    # Gaps and a more cautious master; the oracle follows the reading to rounding.
    N, T, eta, gamma, beta, eps = 64, 400, 0.1, 0.9, 0.999, 1e-8
    a, ts = quad_inputs(N, 3, np.float64)
    one = [0] * T
    th_a, c_a = gap_aware_in_numpy(one, 1, a, ts, eta, gamma, beta, eps, raw_input=False)
    th_b, c_b = gap_aware_in_numpy(one, 1, a, ts, eta, gamma, beta, eps, raw_input=True)
    assert np.array_equal(th_a, th_b) and np.array_equal(c_a, c_b)
    W = 8
    sched = [int(w) for w in oracle.simulate_schedule(W, T, seed=3)]
    th_v, c_v = gap_aware_in_numpy(sched, W, a, ts, eta, gamma, beta, eps, raw_input=False)
    th_g, c_g = gap_aware_in_numpy(sched, W, a, ts, eta, gamma, beta, eps, raw_input=True)
    M = Master(N, W, MODE_GA, Hyper(eta, gamma, beta=beta, eps=eps, f32=False), np.float64)
    M.run_quadratic(np.array(sched, np.uint32), a, ts, seed=0, sigma=0.0)
    assert np.allclose(M.theta, th_v, rtol=1e-9, atol=1e-12)               # the oracle is the reading
    assert np.all(c_v < c_g)                                               # smaller scale C in every coordinate
    ratio = float(np.mean(c_v / c_g))
    apart = float(np.linalg.norm(th_v - th_g) / np.linalg.norm(ts))
    print("mean C (update vector) / C (raw gradient) = %.3f; trajectories apart by %.3f of |theta*| after %d arrivals"
          % (ratio, apart, T))
    assert 0.05 < ratio < 0.95 and 1e-3 < apart < 1.0                      # a real difference, same order of size


# ---------------------------------------------------------------- Gap statistics (App. C.8)
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_gap_statistics_counters_on_dyadic_values(dtype):
    # beta = 1/2, k = 1: 1/(1 - beta^k) = 2; m = 1/32 -> m-hat = 1/16, root 1/4; eps = 0, eta_max = 1/2 -> C = 1/8.
    # |theta - theta^i| in {0, 1/16, 1/8, 1/4, inf, nan} gives Graw in {0, 1/2, 1, 2, inf, nan}: the parameters
    # the paper's form penalises (Graw > 0) are three, those the hinge form penalises (Graw > 1, strictly) one,
    # two are not finite and left out of the sum 1/2 + 1 + 2.
    h = Hyper(eta=0.5, gamma=0.5, beta=0.5, eps=0.0, f32=(dtype == np.float32))
    snap = np.array([3.0, -1.0, 0.5, 2.0, 1.0, 1.0], dtype)
    diff = np.array([0.0, 0.0625, -0.125, 0.25, np.inf, np.nan], dtype)
    theta = (snap + diff).astype(dtype)
    m = np.full(6, 0.03125, dtype)
    r = oracle.gap_statistics(theta, m, snap, 1, h)
    assert (r["n_gt0"], r["n_gt1"], r["n_nonfinite"]) == (3, 1, 2)
    assert r["sum_graw"] == 3.5 and r["mean_graw"] == 3.5 / 6
    assert (r["frac_gt0"], r["frac_gt1"]) == (0.5, 1 / 6)
    # one parameter at a time: each value lands in exactly the expected counters
    expect = [(0, 0, 0, 0.0), (1, 0, 0, 0.5), (1, 0, 0, 1.0), (1, 1, 0, 2.0), (0, 0, 1, 0.0), (0, 0, 1, 0.0)]
    for j, (gt0, gt1, bad, total) in enumerate(expect):
        one = oracle.gap_statistics(theta[j:j + 1], m[j:j + 1], snap[j:j + 1], 1, h)
        assert (one["n_gt0"], one["n_gt1"], one["n_nonfinite"], one["sum_graw"]) == (gt0, gt1, bad, total), j
    # before any arrival (k = 0) m-hat_0 = 0: C = eta_max * eps, here 0, so a zero distance is 0/0 (not finite)
    # and any other distance is infinite
    z = oracle.gap_statistics(theta[:4], m[:4], snap[:4], 0, h)
    assert (z["n_gt0"], z["n_gt1"], z["n_nonfinite"]) == (0, 0, 4)
    # a master's own statistics use its state: after one arrival of worker 0 the Gap of worker 0 is zero everywhere
    M = Master(4, 2, MODE_GA, Hyper(f32=(dtype == np.float32)), dtype)
    M.apply(0, np.array([1.0, -2.0, 0.5, 4.0], dtype))
    own, other = M.gap_statistics(0), M.gap_statistics(1)
    assert (own["n_gt0"], own["sum_graw"]) == (0, 0.0)
    # worker 1 still holds theta_0: distance eta |g|, C_1 = eta (|g| + eps) (Alg. 14 at k = 1), Graw just below 1
    assert (other["n_gt0"], other["n_gt1"], other["n_nonfinite"]) == (4, 0, 0)
    assert abs(other["mean_graw"] - 1.0) < 1e-6


def test_float_tracks_double_on_a_stable_run():
    N, W, T = 2000, 8, 400
    a, ts = quad_inputs(N, 1, np.float32)
    sched = oracle.simulate_schedule(W, T, seed=1)
    for mode in (MODE_SA, MODE_GA):
        M32 = Master(N, W, mode, Hyper(), np.float32)
        M64 = Master(N, W, mode, Hyper(), np.float64)
        M32.run_quadratic(sched, a, ts, seed=1)
        M64.run_quadratic(sched, a.astype(np.float64), ts.astype(np.float64), seed=1)
        rel = np.linalg.norm(M32.theta - M64.theta) / np.linalg.norm(M64.theta)
        assert rel < 1e-4, (mode, rel)


def test_bf16_widening():
    x = ga_inputs.rng(1, 0).standard_normal(1000, dtype=np.float32)
    b = ga_inputs.f32_to_bf16_bits(x)
    w = oracle.bf16_to_f32(b)
    assert np.all(np.abs(w - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(ga_inputs.f32_to_bf16_bits(w), b)        # widening is exact
    assert oracle.bf16_to_f32(np.array([0x3F80, 0xC000, 0x0000], np.uint16)).tolist() == [1.0, -2.0, 0.0]


# ---------------------------------------------------------------- behaviour the paper reports
def test_gap_stays_below_delay_and_penalties_stabilise_momentum():
    # Sec. 4.3 / App. C.8: measured over a run, the mean parameter-wise Gap stays well below the
    # mean delay.  Sec. 2 / 5: with momentum and several workers plain ASGD blows up at a step size
    # where the penalised masters keep descending.  Checked on the synthetic quadratic, W = 8.
    N, W, T, chunk = 4096, 8, 1600, 40
    a, ts = quad_inputs(N, 1, np.float32)
    sched = oracle.simulate_schedule(W, T + 1, seed=1)
    f = lambda th: 0.5 * float(np.sum(a.astype(np.float64) * (th.astype(np.float64) - ts) ** 2))
    f0 = f(np.zeros(N, np.float32))
    loss = {}
    for mode in (MODE_ASGD, MODE_SA, MODE_GA):
        M = Master(N, W, mode, Hyper(), np.float32)
        gaps, taus = [], []
        with np.errstate(all="ignore"):
            for s in range(0, T, chunk):
                taus.append(M.run_quadratic(sched[s:s + chunk], a, ts, seed=1))
                gaps.append(1.0 + M.gap_statistics(int(sched[s + chunk]))["mean_graw"])
        loss[mode] = f(M.theta)
        if mode == MODE_GA:
            mean_tau = float(np.concatenate(taus)[W:].mean())
            assert abs(mean_tau - W) < 0.05                       # steady state: tau averages W
            assert 1.0 < np.mean(gaps) < 0.5 * mean_tau, (np.mean(gaps), mean_tau)
    assert not loss[MODE_ASGD] < f0                               # diverged (or overflowed)
    assert loss[MODE_SA] < 1e-2 * f0 and loss[MODE_GA] < 1e-2 * f0, loss
