"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and its host-only logic (schedule simulator, delay
bookkeeping, per-arrival scalars, argument validation) agrees with the oracle
bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_1909_10802_amd as ga

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "ga.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ga_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert len(names) >= 28
    L = ga.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(ga.SIGNATURES) == names          # the binding covers the whole header
    assert ga.ga_version() == "0.1"


def test_header_is_plain_c_and_usable_from_c(tmp_path):
    import subprocess
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        subprocess.check_call([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-I" + inc, "-fsyntax-only",
                               "-x", "c" if cc == "gcc" else "c++", os.path.join(inc, "ga.h")])
    exe = str(tmp_path / "c_abi_client")
    libdir = os.path.dirname(ga.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-I" + inc,
                           os.path.join(ROOT, "tests", "c_abi_client.c"), "-o", exe, "-L" + libdir, "-lga",
                           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0 and "c client ok" in out.stdout, out.stdout


def test_struct_layouts_match_the_header():
    assert C.sizeof(ga.ga_arrival) == 16 and ga.ARRIVAL_DTYPE.itemsize == 16
    assert C.sizeof(ga.ga_diag) == 32
    assert ga.ga_grad_source.dev_a.offset == 8 and ga.ga_grad_source.seed.offset == 24
    assert C.sizeof(ga.ga_config) == 80 and ga.ga_config.eta.offset == 20 and ga.ga_config.track_gap.offset == 48
    cfg = ga.ga_config_init()
    assert (cfg.family, cfg.mode, cfg.track_gap, cfg.gap_scope, cfg.n_layers, cfg.host_layer_sizes) == (0, 3, 0, 0, 0, None)
    assert np.allclose([cfg.eta, cfg.gamma, cfg.beta, cfg.eps, cfg.adam_beta1, cfg.adam_beta2, cfg.adam_eps],
                       [0.1, 0.9, 0.999, 1e-8, 0.9, 0.999, 1e-8], rtol=1e-6)


@pytest.mark.parametrize("dist,sigma", [(ga.GA_DIST_EXP, 1.0), (ga.GA_DIST_LOGNORMAL, 1.0), (ga.GA_DIST_HETERO, 1.5)])
def test_schedule_simulator_matches_oracle(dist, sigma):
    for W, T, seed in [(1, 50, 0), (8, 1000, 1), (32, 10000, 2), (128, 5000, 2**40 + 17)]:
        mine = ga.ga_simulate_schedule(W, T, dist, sigma, seed)
        ref = oracle.simulate_schedule(W, T, dist, sigma, seed)
        assert np.array_equal(mine, ref), (W, T, seed)


def test_delays_match_oracle_and_resume():
    W, T = 16, 3000
    sched = ga.ga_simulate_schedule(W, T, seed=5)
    tau, it = ga.ga_delays_from_schedule(W, sched)
    tau_o, it_o = oracle.delays(W, sched)
    assert np.array_equal(tau, tau_o) and np.array_equal(it, it_o)
    ta, ia = ga.ga_delays_from_schedule(W, sched[:1000])
    tb, ib = ga.ga_delays_from_schedule(W, sched[1000:], k0=1000, host_iter=ia.copy())
    assert np.array_equal(np.concatenate([ta, tb]), tau) and np.array_equal(ib, it)


@pytest.mark.parametrize("mode", [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_SA_STEP, ga.GA_MODE_GA])
def test_arrival_rows(mode):
    W, T, eta, beta = 8, 500, np.float32(0.1), np.float32(0.999)
    sched = ga.ga_simulate_schedule(W, T, seed=3)
    it = np.zeros(W, dtype=np.uint64)
    rows = ga.ga_plan_arrivals(W, sched, 0, it, mode, float(eta), float(beta))
    tau_o, it_o = oracle.delays(W, sched)
    assert np.array_equal(rows["worker"], sched)
    assert np.array_equal(rows["tau"], tau_o.astype(np.float32))
    assert np.array_equal(it, it_o)
    lr = eta / tau_o.astype(np.float32) if mode == ga.GA_MODE_SA_STEP else np.full(T, eta)
    assert np.array_equal(rows["lr"], lr.astype(np.float32))
    k = np.arange(1, T + 1)
    with np.errstate(divide="ignore"):
        inv = (1.0 / (1.0 - np.float64(beta) ** (k - 1).astype(np.float64))).astype(np.float32)
    inv[0] = 0.0                                        # before the first arrival m-hat is taken as 0
    assert np.array_equal(rows["inv_bc_prev"], inv)
    # continuing from step 200 gives the same rows as the tail of the full plan
    it2 = oracle.delays(W, sched[:200])[1]
    rows2 = ga.ga_plan_arrivals(W, sched[200:], 200, it2, mode, float(eta), float(beta))
    assert np.array_equal(rows2, rows[200:])


def test_host_argument_errors():
    with pytest.raises(ga.GaError) as e:
        ga.ga_simulate_schedule(0, 10)
    assert e.value.status == ga.GA_ERR_ARG
    with pytest.raises(ga.GaError):
        ga.ga_simulate_schedule(4, 10, dist=7)
    with pytest.raises(ga.GaError) as e:
        ga.ga_delays_from_schedule(4, np.array([0, 1, 4], dtype=np.uint32))
    assert e.value.status == ga.GA_ERR_WORKER
    with pytest.raises(ga.GaError):
        ga.ga_delays_from_schedule(2, np.array([0, 1], dtype=np.uint32), k0=3, host_iter=np.array([5, 0], np.uint64))
    with pytest.raises(ga.GaError):
        ga.ga_plan_arrivals(2, np.array([0, 1], dtype=np.uint32), 0, np.zeros(2, np.uint64), 9, 0.1, 0.999)
    with pytest.raises(ga.GaError):
        ga.ga_plan_arrivals(2, np.array([0, 1], dtype=np.uint32), 0, np.zeros(2, np.uint64), 0, 0.1, 1.0)


def test_workspace_size_and_create_validation():
    L = ga.lib()
    assert ga.ga_workspace_bytes(0, 4) == 0 and ga.ga_workspace_bytes(4, 0) == 0
    n1 = ga.ga_workspace_bytes(1, 1)
    assert n1 % 256 == 0 and n1 >= 4 * 256
    big = ga.ga_workspace_bytes(350_000_000, 128)
    assert big >= 131 * 350_000_000 * 4 and big < 131 * 350_000_064 * 4 + (1 << 20) + 3 * 8192 * 4
    # the W snapshot rows are padded to 64 floats; theta, v, m are interleaved by tiles of 8192 floats
    assert ga.ga_workspace_bytes(65, 3) - ga.ga_workspace_bytes(64, 3) == 3 * 64 * 4
    assert ga.ga_workspace_bytes(8193, 3) - ga.ga_workspace_bytes(8192, 3) == 3 * 8192 * 4 + 3 * 64 * 4

    ctx = C.c_void_p()
    fake = C.c_void_p(0x7F0000000000)               # never dereferenced: validation fails first

    def create(N=100, W=2, eta=0.1, gamma=0.9, mode=ga.GA_MODE_GA, ws=fake, nbytes=1 << 30):
        return L.ga_create(C.byref(ctx), N, W, eta, gamma, mode, ws, nbytes, None)

    assert create(N=0) == ga.GA_ERR_ARG
    assert create(W=0) == ga.GA_ERR_ARG
    assert create(eta=0.0) == ga.GA_ERR_ARG and create(eta=-1.0) == ga.GA_ERR_ARG
    assert create(eta=float("nan")) == ga.GA_ERR_ARG
    assert create(gamma=1.0) == ga.GA_ERR_ARG and create(gamma=-1.0) == ga.GA_ERR_ARG
    assert create(mode=5) == ga.GA_ERR_ARG and create(mode=-1) == ga.GA_ERR_ARG
    assert create(ws=None) == ga.GA_ERR_ARG
    assert create(ws=C.c_void_p(0x7F0000000010)) == ga.GA_ERR_ALIGN
    assert create(nbytes=1024) == ga.GA_ERR_ALIGN
    assert b"workspace" in L.ga_last_error(None)
    assert L.ga_create(None, 100, 2, 0.1, 0.9, 3, fake, 1 << 30, None) == ga.GA_ERR_ARG
    assert ctx.value is None
    # null context is an argument error everywhere, never a crash
    assert L.ga_apply(None, 0, fake, 0) == ga.GA_ERR_ARG
    assert L.ga_set_lr(None, 0.1) == ga.GA_ERR_ARG
    assert L.ga_get_theta(None, fake) == ga.GA_ERR_ARG
    assert L.ga_step(None) == 0
    L.ga_destroy(None)


def test_warmup_schedule():
    # App. C.5: start at eta / N, reach eta linearly at the end of the warm-up, constant afterwards
    eta, W, steps = np.float32(0.1), 8, 50
    lr = ga.ga_warmup_lr(float(eta), W, steps, 0, 80)
    k = np.arange(1, 81, dtype=np.float64)
    lo = float(eta) / W
    expect = np.where(k < steps, lo + (float(eta) - lo) * k / steps, float(eta)).astype(np.float32)
    assert np.array_equal(lr, expect)
    assert lr[0] > lo and np.all(np.diff(lr[:steps]) > 0) and np.all(lr[steps - 1:] == eta)
    assert np.array_equal(ga.ga_warmup_lr(float(eta), W, steps, 30, 50), lr[30:])
    with pytest.raises(ga.GaError):
        ga.ga_warmup_lr(0.0, W, steps, 0, 4)


def test_bookkeeping_matches_oracle_on_random_schedules():
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None)
    @given(st.integers(1, 40), st.lists(st.integers(0, 10_000), min_size=0, max_size=300), st.integers(0, 1000),
           st.sampled_from([ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_SA_STEP, ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE]))
    def check(W, raw, k0, mode):
        sched = (np.array(raw, dtype=np.uint64) % W).astype(np.uint32)
        rng = np.random.default_rng(len(raw) + W)
        it0 = rng.integers(0, k0 + 1, W).astype(np.uint64)
        tau, it = ga.ga_delays_from_schedule(W, sched, k0, it0.copy())
        tau_o, it_o = oracle.delays(W, sched, k0, it0.copy())
        assert np.array_equal(tau, tau_o) and np.array_equal(it, it_o)
        rows = ga.ga_plan_arrivals(W, sched, k0, it0.copy(), mode, 0.05, 0.99)
        assert np.array_equal(rows["tau"], tau_o.astype(np.float32)) and np.array_equal(rows["worker"], sched)
        assert np.all(tau_o >= 1)

    check()


def test_oracle_is_clean_under_address_and_undefined_sanitizers(tmp_path):
    # host code only: the oracle rebuilt with -fsanitize and driven through a short trajectory of every master
    import subprocess
    import sys
    lib = str(tmp_path / "libga_oracle_san.so")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-o", lib,
                           os.path.join(ROOT, "oracle", "ga_oracle.cpp")])
    script = r'''
import sys, numpy as np
sys.path.insert(0, %r)
import oracle
oracle._LIB = %r
oracle.build = lambda force=False: oracle._LIB
N, W, T = 1003, 5, 60
a = np.linspace(0.1, 1, N).astype(np.float32); ts = np.cos(np.arange(N)).astype(np.float32)
sched = oracle.simulate_schedule(W, T, oracle.DIST_HETERO, 1.5, 3)
for cls, kw in [(oracle.Master, {}), (oracle.Master, {"nesterov": True}), (oracle.DanaMaster, {}), (oracle.AdamMaster, {})]:
    for mode in (oracle.MODE_SA, oracle.MODE_GA, oracle.MODE_GA_HINGE):
        M = cls(N, W, mode, oracle.Hyper(0.01, 0.9), **kw)
        M.run_quadratic(sched, a, ts, 7)
        M.gap_statistics(1)
L = oracle.LayerwiseMaster(N, W, oracle.MODE_GA, oracle.Hyper(), [3, 500, 500])
L.run_quadratic(sched, a, ts, 7)
oracle.simulate_schedule_gamma(8, 200, oracle.DIST_GAMMA_HETERO, 1, 128.0, 0.6, 0.1)
oracle.speedup_times(4, 50, oracle.DIST_GAMMA_HOMO, 1)
oracle.box_muller_raw(np.arange(100, dtype=np.uint32) << np.uint32(9), np.arange(100, dtype=np.uint32) * np.uint32(40503))
print("sanitized oracle ok")
''' % (ROOT, lib)
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    ubsan = subprocess.check_output(["gcc", "-print-file-name=libubsan.so"], text=True).strip()
    env = dict(os.environ, LD_PRELOAD=asan + " " + ubsan, ASAN_OPTIONS="detect_leaks=0")
    out = subprocess.run([sys.executable, "-c", script], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert out.returncode == 0 and "sanitized oracle ok" in out.stdout, out.stdout[-3000:]
