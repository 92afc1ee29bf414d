"""ctypes loader for the CPU oracle (oracle/ga_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing here touches the GPU library, and the
GPU library never imports this package.

The wrappers only marshal numpy arrays; all arithmetic is in the C++ file.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ga_oracle.cpp")
_LIB = os.path.join(_HERE, "libga_oracle.so")

MODE_ASGD, MODE_SA, MODE_SA_STEP, MODE_GA, MODE_GA_HINGE = range(5)
DIST_EXP, DIST_LOGNORMAL, DIST_HETERO, DIST_GAMMA_HOMO, DIST_GAMMA_HETERO = range(5)

CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared"]


def build(force=False):
    """Compile the oracle with g++ (floating-point contraction off)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", *CXXFLAGS, "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _declare(_lib)
    return _lib


_u64, _u32, _f64, _int = C.c_uint64, C.c_uint32, C.c_double, C.c_int
_p = C.c_void_p


def _declare(L):
    L.orc_noise_z_f32.restype = C.c_float
    L.orc_noise_z_f32.argtypes = [_u64, _u64, _u64]
    L.orc_noise_z_ref.restype = _f64
    L.orc_noise_z_ref.argtypes = [_u64, _u64, _u64]
    L.orc_noise_fill_f32.argtypes = [_u64, _u64, _u64, _u64, _p]
    L.orc_noise_fill_ref.argtypes = [_u64, _u64, _u64, _u64, _p]
    L.orc_philox4x32_10.argtypes = [_p, _p, _p]
    L.orc_box_muller_raw.argtypes = [_p, _p, _u64, _p, _p]
    L.orc_iteration_time.restype = _f64
    L.orc_iteration_time.argtypes = [_int, _f64, _u64, _u32, _u64]
    L.orc_simulate_schedule.argtypes = [_u32, _u64, _int, _f64, _u64, _p, _p]
    L.orc_iteration_time_gamma.restype = _f64
    L.orc_iteration_time_gamma.argtypes = [_int, _f64, _f64, _f64, _u64, _u32, _u64]
    L.orc_gamma_draw.restype = _f64
    L.orc_gamma_draw.argtypes = [_f64, _f64, _u64, _u64]
    L.orc_simulate_schedule_gamma.argtypes = [_u32, _u64, _int, _f64, _f64, _f64, _u64, _p, _p]
    L.orc_speedup_times.argtypes = [_u32, _u64, _int, _f64, _f64, _f64, _u64, _p, _p]
    L.orc_schedule_from_times.argtypes = [_u32, _u64, _p, _u64, _p]
    L.orc_delays.argtypes = [_u32, _u64, _p, _u64, _p, _p]
    hyp = [_f64] * 5
    for sfx in ("f32", "f64"):
        getattr(L, "orc_step_" + sfx).argtypes = [_u64, _p, _p, _p, _p, _p, _int, _u64, _u64, *hyp, _int]
        getattr(L, "orc_step_nag_" + sfx).argtypes = [_u64, _p, _p, _p, _p, _p, _int, _u64, _u64, *hyp, _int]
        getattr(L, "orc_dana_step_" + sfx).argtypes = [_u64, _p, _p, _p, _p, _p, _p, _int, _u64, _u64, *hyp, _int]
        getattr(L, "orc_adam_step_" + sfx).argtypes = [_u64, _p, _p, _p, _p, _p, _p, _int, _u64, _u64,
                                                       _f64, _f64, _f64, _f64, _f64, _f64, _f64, _int]
        getattr(L, "orc_step_layerwise_" + sfx).argtypes = [_u64, _p, _p, _p, _p, _p, _p, _u32, _int, _u64, *hyp, _p, _int]
        getattr(L, "orc_quadratic_gradient_" + sfx).argtypes = [_u64, _p, _p, _p, _p, _p, _u64, _u64, _f64]
        getattr(L, "orc_gap_statistics_" + sfx).argtypes = [_u64, _p, _p, _p, _u64, _f64, _f64, _f64, _p, _p, _p, _p]
        getattr(L, "orc_run_quadratic_" + sfx).argtypes = [
            _u64, _u32, _u64, _p, _p, _p, _p, _p, _p, _p, _p, _u64, _f64, _int, *hyp, _int, _p, _p, _p]
        getattr(L, "orc_run_buffers_" + sfx).argtypes = [
            _u64, _u32, _u64, _p, _p, _p, _p, _p, _p, _u32, _int, _int, *hyp, _int, _p, _p, _p]
    L.orc_num_threads.restype = _int
    L.orc_set_num_threads.argtypes = [_int]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _chk(a, dtype, n=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    if n is not None:
        assert a.size == n, (a.size, n)
    return a


def _sfx(dtype):
    dtype = np.dtype(dtype)
    assert dtype in (np.float32, np.float64)
    return "f32" if dtype == np.float32 else "f64"


# ------------------------------------------------------------------ generators
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def noise_f32(seed, k, j0, n):
    out = np.empty(n, dtype=np.float32)
    lib().orc_noise_fill_f32(seed, k, j0, n, _ptr(out))
    return out


def box_muller_raw(xa, xb):
    """(r cos, r sin) of the noise transform for raw Philox word pairs."""
    xa, xb = _chk(np.ascontiguousarray(xa), np.uint32), _chk(np.ascontiguousarray(xb), np.uint32)
    zc, zs = np.empty(xa.size, np.float32), np.empty(xa.size, np.float32)
    lib().orc_box_muller_raw(_ptr(xa), _ptr(xb), xa.size, _ptr(zc), _ptr(zs))
    return zc, zs


def noise_ref(seed, k, j0, n):
    out = np.empty(n, dtype=np.float64)
    lib().orc_noise_fill_ref(seed, k, j0, n, _ptr(out))
    return out


def iteration_time(dist, sigma, seed, w, n):
    return lib().orc_iteration_time(dist, sigma, seed, w, n)


def simulate_schedule(W, T, dist=DIST_EXP, sigma=1.0, seed=0, with_times=False):
    sched = np.empty(T, dtype=np.uint32)
    times = np.empty(T, dtype=np.float64) if with_times else None
    rc = lib().orc_simulate_schedule(W, T, dist, sigma, seed, _ptr(sched), _ptr(times))
    assert rc == 0
    return (sched, times) if with_times else sched


def gamma_draw(alpha, scale, seed, n):
    return lib().orc_gamma_draw(alpha, scale, seed, n)


def iteration_time_gamma(dist, seed, w, n, mean=128.0, v_mach=0.1, v_task=0.1):
    return lib().orc_iteration_time_gamma(dist, mean, v_mach, v_task, seed, w, n)


def simulate_schedule_gamma(W, T, dist, seed=0, mean=128.0, v_mach=0.1, v_task=0.1, with_times=False):
    """Arrival schedule under the gamma model of App. C.3 (Alg. 12: DIST_GAMMA_HOMO, Alg. 13: DIST_GAMMA_HETERO)."""
    sched = np.empty(T, dtype=np.uint32)
    times = np.empty(T, dtype=np.float64) if with_times else None
    rc = lib().orc_simulate_schedule_gamma(W, T, dist, mean, v_mach, v_task, seed, _ptr(sched), _ptr(times))
    assert rc == 0
    return (sched, times) if with_times else sched


def speedup_times(W, iters, dist, seed=0, mean=128.0, v_mach=0.1, v_task=0.1):
    """(ASGD wall time, SSGD wall time) to process W*iters batches (App. D)."""
    a, s = C.c_double(), C.c_double()
    rc = lib().orc_speedup_times(W, iters, dist, mean, v_mach, v_task, seed, C.byref(a), C.byref(s))
    assert rc == 0
    return a.value, s.value


def schedule_from_times(times, T):
    times = np.ascontiguousarray(times, dtype=np.float64)
    W, max_iters = times.shape
    sched = np.empty(T, dtype=np.uint32)
    rc = lib().orc_schedule_from_times(W, T, _ptr(times), max_iters, _ptr(sched))
    assert rc == 0, "time table too short"
    return sched


def delays(W, schedule, k0=0, iter_=None):
    """Return (tau[T], iter[W]) after replaying the schedule from step k0."""
    schedule = _chk(np.ascontiguousarray(schedule, dtype=np.uint32), np.uint32)
    it = np.zeros(W, dtype=np.uint64) if iter_ is None else _chk(iter_, np.uint64, W)
    tau = np.empty(schedule.size, dtype=np.uint64)
    lib().orc_delays(W, schedule.size, _ptr(schedule), k0, _ptr(it), _ptr(tau))
    return tau, it


# ------------------------------------------------------------------ master
class Hyper:
    """Hyper-parameters of the master (Alg. 2-5, 14). Defaults: App. C.4, C.6."""

    def __init__(self, eta=0.1, gamma=0.9, eta_max=None, beta=0.999, eps=1e-8, eta_k=None, f32=True):
        r = (lambda x: float(np.float32(x))) if f32 else float
        self.eta_max = r(eta if eta_max is None else eta_max)
        self.eta_k = r(eta if eta_k is None else eta_k)
        self.gamma = r(gamma)
        self.beta = r(beta)
        self.eps = r(eps)

    def args(self):
        return (self.eta_k, self.eta_max, self.gamma, self.beta, self.eps)


def step(theta, v, m, snap_i, g, mode, k, tau, hyper, track_gap=False, nesterov=False):
    """One arrival, in place on theta, v, m, snap_i."""
    s = _sfx(theta.dtype)
    n = theta.size
    for a in (theta, v, m, snap_i, g):
        _chk(a, theta.dtype, n)
    getattr(lib(), ("orc_step_nag_" if nesterov else "orc_step_") + s)(n, _ptr(theta), _ptr(v), _ptr(m), _ptr(snap_i), _ptr(g), mode, k, tau,
                                    *hyper.args(), int(track_gap))


def quadratic_gradient(snap_i, a, theta_star, seed, k, sigma=0.01, idx=None):
    s = _sfx(snap_i.dtype)
    n = snap_i.size
    g = np.empty(n, dtype=snap_i.dtype)
    if idx is not None:
        idx = _chk(idx, np.uint64, n)
    getattr(lib(), "orc_quadratic_gradient_" + s)(n, _ptr(g), _ptr(snap_i), _ptr(_chk(a, snap_i.dtype, n)),
                                                  _ptr(_chk(theta_star, snap_i.dtype, n)), _ptr(idx), seed, k, sigma)
    return g


def gap_statistics(theta, m, snap_i, k, hyper):
    """Returns dict(mean_graw, frac_gt1, frac_gt0, n_nonfinite, sum_graw)."""
    s = _sfx(theta.dtype)
    n = theta.size
    sm = C.c_double()
    gt1, gt0, bad = C.c_uint64(), C.c_uint64(), C.c_uint64()
    getattr(lib(), "orc_gap_statistics_" + s)(n, _ptr(theta), _ptr(_chk(m, theta.dtype, n)),
                                              _ptr(_chk(snap_i, theta.dtype, n)), k, hyper.beta, hyper.eta_max,
                                              hyper.eps, C.byref(sm), C.byref(gt1), C.byref(gt0), C.byref(bad))
    return dict(sum_graw=sm.value, mean_graw=sm.value / n if n else 0.0, frac_gt1=gt1.value / n if n else 0.0,
                frac_gt0=gt0.value / n if n else 0.0, n_gt1=gt1.value, n_gt0=gt0.value, n_nonfinite=bad.value)


class Master:
    """State of one parameter-server master, advanced by the oracle routines."""

    def __init__(self, N, W, mode, hyper, dtype=np.float32, theta0=None, track_gap=False, nesterov=False):
        self.N, self.W, self.mode, self.hyper, self.dtype = N, W, mode, hyper, np.dtype(dtype)
        self.track_gap = track_gap
        self.nesterov = nesterov
        self.theta = np.zeros(N, dtype) if theta0 is None else np.array(theta0, dtype=dtype)
        self.v = np.zeros(N, dtype)
        self.m = np.zeros(N, dtype)
        self.snaps = np.tile(self.theta, (W, 1))       # theta^i = theta_0 for every worker
        self.iter = np.zeros(W, dtype=np.uint64)
        self.k = 0
        self.tau_log = []

    def apply(self, worker, g):
        self.k += 1
        tau = self.k - int(self.iter[worker])
        step(self.theta, self.v, self.m, self.snaps[worker], np.ascontiguousarray(g, dtype=self.dtype), self.mode,
             self.k, tau, self.hyper, self.track_gap, self.nesterov)
        self.iter[worker] = self.k
        self.tau_log.append(tau)
        return tau

    def run_quadratic(self, schedule, a, theta_star, seed, sigma=0.01, idx=None):
        if self.nesterov:                               # arrival by arrival (the C loop is heavy-ball only)
            for w in schedule:
                w = int(w)
                self.apply(w, quadratic_gradient(self.snaps[w], a, theta_star, seed, self.k + 1, sigma, idx))
            return np.array(self.tau_log[-len(schedule):], dtype=np.uint64)
        s = _sfx(self.dtype)
        schedule = _chk(np.ascontiguousarray(schedule, dtype=np.uint32), np.uint32)
        T = schedule.size
        tau = np.empty(T, dtype=np.uint64)
        kio = C.c_uint64(self.k)
        if idx is not None:
            idx = _chk(idx, np.uint64, self.N)
        getattr(lib(), "orc_run_quadratic_" + s)(
            self.N, self.W, T, _ptr(schedule), _ptr(self.theta), _ptr(self.v), _ptr(self.m), _ptr(self.snaps),
            _ptr(_chk(a, self.dtype, self.N)), _ptr(_chk(theta_star, self.dtype, self.N)), _ptr(idx), seed, sigma,
            self.mode, *self.hyper.args(), int(self.track_gap), C.byref(kio), _ptr(self.iter), _ptr(tau))
        self.k = kio.value
        self.tau_log.extend(int(t) for t in tau)
        return tau

    def run_buffers(self, schedule, bufs, pick_by_worker=True):
        if self.nesterov:
            for w in schedule:
                w = int(w)
                self.apply(w, bufs[w % len(bufs)] if pick_by_worker else bufs[self.k % len(bufs)])
            return np.array(self.tau_log[-len(schedule):], dtype=np.uint64)
        s = _sfx(self.dtype)
        schedule = _chk(np.ascontiguousarray(schedule, dtype=np.uint32), np.uint32)
        T = schedule.size
        bufs = _chk(bufs, self.dtype)
        assert bufs.ndim == 2 and bufs.shape[1] == self.N
        tau = np.empty(T, dtype=np.uint64)
        kio = C.c_uint64(self.k)
        getattr(lib(), "orc_run_buffers_" + s)(
            self.N, self.W, T, _ptr(schedule), _ptr(self.theta), _ptr(self.v), _ptr(self.m), _ptr(self.snaps),
            _ptr(bufs), bufs.shape[0], int(pick_by_worker), self.mode, *self.hyper.args(), int(self.track_gap),
            C.byref(kio), _ptr(self.iter), _ptr(tau))
        self.k = kio.value
        self.tau_log.extend(int(t) for t in tau)
        return tau

    def gap_statistics(self, worker):
        return gap_statistics(self.theta, self.m, self.snaps[worker], self.k, self.hyper)


class LayerwiseMaster(Master):
    """Gap-Aware master with one Gap per layer (Eq. 4); a single layer gives the global Gap (Def. 1)."""

    def __init__(self, N, W, mode, hyper, layer_sizes=None, dtype=np.float32, theta0=None, nesterov=False):
        super().__init__(N, W, mode, hyper, dtype, theta0, nesterov=nesterov)
        assert mode in (MODE_GA, MODE_GA_HINGE)
        self.layer_sizes = np.array([N] if layer_sizes is None else layer_sizes, dtype=np.uint64)
        assert int(self.layer_sizes.sum()) == N
        self.last_gaps = np.zeros(self.layer_sizes.size, self.dtype)

    def apply(self, worker, g):
        self.k += 1
        tau = self.k - int(self.iter[worker])
        g = np.ascontiguousarray(g, dtype=self.dtype)
        rc = getattr(lib(), "orc_step_layerwise_" + _sfx(self.dtype))(
            self.N, _ptr(self.theta), _ptr(self.v), _ptr(self.m), _ptr(self.snaps[worker]),
            _ptr(_chk(g, self.dtype, self.N)), _ptr(self.layer_sizes), self.layer_sizes.size, self.mode, self.k,
            *self.hyper.args(), _ptr(self.last_gaps), int(self.nesterov))
        assert rc == 0
        self.iter[worker] = self.k
        self.tau_log.append(tau)
        return tau

    def run_quadratic(self, schedule, a, theta_star, seed, sigma=0.01, idx=None):
        for w in schedule:
            w = int(w)
            self.apply(w, quadratic_gradient(self.snaps[w], a, theta_star, seed, self.k + 1, sigma, idx))

    def run_buffers(self, schedule, bufs, pick_by_worker=True):
        for w in schedule:
            w = int(w)
            self.apply(w, bufs[w % len(bufs)] if pick_by_worker else bufs[self.k % len(bufs)])


class DanaMaster:
    """DANA / DANA-SA / DANA-GA master (Alg. 6-8): per-worker momenta v^i, their running sum,
    look-ahead snapshots.  The arrival loop is driven from Python, one oracle step per arrival."""

    def __init__(self, N, W, mode, hyper, dtype=np.float32, theta0=None, track_gap=False):
        self.N, self.W, self.mode, self.hyper, self.dtype = N, W, mode, hyper, np.dtype(dtype)
        self.track_gap = track_gap
        self.theta = np.zeros(N, dtype) if theta0 is None else np.array(theta0, dtype=dtype)
        self.vw = np.zeros((W, N), dtype)                # v^i
        self.vsum = np.zeros(N, dtype)                   # sum_j v^j
        self.m = np.zeros(N, dtype)
        self.snaps = np.tile(self.theta, (W, 1))         # theta^i = theta_0
        self.iter = np.zeros(W, dtype=np.uint64)
        self.k = 0
        self.tau_log = []

    def apply(self, worker, g):
        self.k += 1
        tau = self.k - int(self.iter[worker])
        g = np.ascontiguousarray(g, dtype=self.dtype)
        getattr(lib(), "orc_dana_step_" + _sfx(self.dtype))(
            self.N, _ptr(self.theta), _ptr(self.vw[worker]), _ptr(self.vsum), _ptr(self.m), _ptr(self.snaps[worker]),
            _ptr(_chk(g, self.dtype, self.N)), self.mode, self.k, tau, *self.hyper.args(), int(self.track_gap))
        self.iter[worker] = self.k
        self.tau_log.append(tau)
        return tau

    def run_quadratic(self, schedule, a, theta_star, seed, sigma=0.01, idx=None):
        for w in schedule:
            w = int(w)
            self.apply(w, quadratic_gradient(self.snaps[w], a, theta_star, seed, self.k + 1, sigma, idx))

    def run_buffers(self, schedule, bufs, pick_by_worker=True):
        for w in schedule:
            w = int(w)
            self.apply(w, bufs[w % len(bufs)] if pick_by_worker else bufs[self.k % len(bufs)])

    def gap_statistics(self, worker):
        return gap_statistics(self.theta, self.m, self.snaps[worker], self.k, self.hyper)


class AdamMaster:
    """Adam / Adam-SA / Adam-GA master (Alg. 9-11).  c is the Alg. 14 state of the update vector."""

    def __init__(self, N, W, mode, hyper, dtype=np.float32, theta0=None, track_gap=False, beta1=0.9, beta2=0.999,
                 adam_eps=1e-8):
        self.N, self.W, self.mode, self.hyper, self.dtype = N, W, mode, hyper, np.dtype(dtype)
        self.track_gap = track_gap
        r = (lambda x: float(np.float32(x))) if self.dtype == np.float32 else float
        self.beta1, self.beta2, self.adam_eps = r(beta1), r(beta2), r(adam_eps)
        self.theta = np.zeros(N, dtype) if theta0 is None else np.array(theta0, dtype=dtype)
        self.m1 = np.zeros(N, dtype)
        self.v2 = np.zeros(N, dtype)
        self.m = np.zeros(N, dtype)                      # Alg. 14 state (called c in the C++ file)
        self.snaps = np.tile(self.theta, (W, 1))
        self.iter = np.zeros(W, dtype=np.uint64)
        self.k = 0
        self.tau_log = []

    def apply(self, worker, g):
        self.k += 1
        tau = self.k - int(self.iter[worker])
        g = np.ascontiguousarray(g, dtype=self.dtype)
        h = self.hyper
        getattr(lib(), "orc_adam_step_" + _sfx(self.dtype))(
            self.N, _ptr(self.theta), _ptr(self.m1), _ptr(self.v2), _ptr(self.m), _ptr(self.snaps[worker]),
            _ptr(_chk(g, self.dtype, self.N)), self.mode, self.k, tau, h.eta_k, h.eta_max, h.beta, h.eps,
            self.beta1, self.beta2, self.adam_eps, int(self.track_gap))
        self.iter[worker] = self.k
        self.tau_log.append(tau)
        return tau

    run_quadratic = DanaMaster.run_quadratic
    run_buffers = DanaMaster.run_buffers
    gap_statistics = DanaMaster.gap_statistics


def num_threads():
    return lib().orc_num_threads()


def set_num_threads(n):
    lib().orc_set_num_threads(int(n))


def bf16_to_f32(u16):
    """Widen bfloat16 bit patterns (uint16) to float32: the bits move to the top half."""
    u16 = _chk(np.ascontiguousarray(u16), np.uint16)
    return (u16.astype(np.uint32) << np.uint32(16)).view(np.float32)
