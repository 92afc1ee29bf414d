"""The library's kernels on a CPU.  The kernel sources (csrc/*.hip) are compiled as ordinary C++ through a stand-in
for the HIP device header (tests/cpu_device/shim) and run one fiber per GPU thread, block after block, together with
the real host code, under AddressSanitizer and UndefinedBehaviorSanitizer.  Every load and store of every kernel is
therefore bounds-checked on launch shapes with ragged tails, and the state after a schedule is compared with the
oracle: the arithmetic is IEEE float operations in a fixed order on both targets, so the comparison is bit for bit
(sums of many terms, i.e. the Gap statistics and the layer norms, to 1e-6).  This finds indexing mistakes before
they can fault a GPU; it does not replace the GPU tests, which run the code the product runs."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import ga_inputs
import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "cpu_device")
CSRC = os.path.join(ROOT, "paper_1909_10802_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang++"
FLAGS = ["-std=c++17", "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(HERE, "shim"), "-I/opt/rocm/include",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
         # locals of a fiber outlive its switches: the use-after-return machinery of ASan does not follow that
         "-fsanitize-address-use-after-return=never",
         "-gline-tables-only", "-O0", "-Wall", "-Wextra", "-Werror"]
KERNEL_SOURCES = ["ga_apply.hip", "ga_persistent.hip", "ga_batched.hip", "ga_layerwise.hip", "ga_aux.hip"]
HOST_SOURCES = [os.path.join(CSRC, "ga_host.cpp"), os.path.join(HERE, "cpu_device.cpp"), os.path.join(HERE, "driver.cpp"),
                os.path.join(HERE, "probe_stand_ins.cpp"), os.path.join(ROOT, "tests", "host_sim", "fake_runtime.cpp")]

pytestmark = pytest.mark.skipif(not os.path.exists(CLANG), reason="needs the ROCm clang++")

MODE = {0: oracle.MODE_ASGD, 1: oracle.MODE_SA, 2: oracle.MODE_SA_STEP, 3: oracle.MODE_GA, 4: oracle.MODE_GA_HINGE}


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("cpu_device")
    jobs = []
    for src in KERNEL_SOURCES:
        jobs.append([CLANG, *FLAGS, "-x", "c++", "-c", os.path.join(CSRC, src), "-o", str(out / (src + ".o"))])
    for src in HOST_SOURCES:
        jobs.append([CLANG, *FLAGS, "-c", src, "-o", str(out / (os.path.basename(src) + ".o"))])

    def compile_one(cmd):
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-4000:]
    with ThreadPoolExecutor(max_workers=8) as pool:
        list(pool.map(compile_one, jobs))
    exe = str(out / "driver")
    subprocess.check_call([CLANG, "-fsanitize=address,undefined", *[j[-1] for j in jobs], "-o", exe])
    return exe


def run(driver, tmp_path, N, W, T, seed, family=0, mode=3, source=0, scope=0, layers=None, nesterov=0, track_gap=0,
        bf16=0, n_bufs=3, pick=0, queue=0, resident_bytes=240 << 20, eta=0.1, gamma=0.9, sigma=0.02, static_diag=0,
        theta0=False):
    """Runs one scenario in the CPU build and the same in the oracle; returns (state arrays of the build, oracle)."""
    d = str(tmp_path)
    sched = oracle.simulate_schedule(W, T, oracle.DIST_EXP, 0.7, seed)
    sched.astype(np.uint32).tofile(os.path.join(d, "sched.bin"))
    diag_worker = int(sched[-2]) if W > 1 and sched[-2] != sched[-1] else int((sched[-1] + 1) % W)
    hy = oracle.Hyper(eta, 0.0 if family == 2 else gamma)
    start = None
    if theta0:
        start = ga_inputs.optimum(N, seed + 1)
        start.tofile(os.path.join(d, "theta0.bin"))
    if scope:
        sizes = [N] if scope == 2 else layers
        np.array(sizes, np.uint64).tofile(os.path.join(d, "layers.bin"))
        O = oracle.LayerwiseMaster(N, W, MODE[mode], hy, layer_sizes=sizes, nesterov=bool(nesterov), theta0=start)
    elif family == 0:
        O = oracle.Master(N, W, MODE[mode], hy, track_gap=bool(track_gap), nesterov=bool(nesterov), theta0=start)
    elif family == 1:
        O = oracle.DanaMaster(N, W, MODE[mode], hy, track_gap=bool(track_gap), theta0=start)
    else:
        O = oracle.AdamMaster(N, W, MODE[mode], hy, track_gap=bool(track_gap), theta0=start)
    if source <= 1:
        a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
        a.tofile(os.path.join(d, "a.bin")); ts.tofile(os.path.join(d, "ts.bin"))
        O.run_quadratic(sched, a, ts, seed, sigma=sigma)
    else:
        bufs = ga_inputs.gradient_buffers(n_bufs, N, seed=seed, std=0.3)
        if bf16:
            bits = ga_inputs.f32_to_bf16_bits(bufs).reshape(n_bufs, N)
            bits.tofile(os.path.join(d, "bufs.bin"))
            ref = oracle.bf16_to_f32(bits).reshape(n_bufs, N)
        else:
            bufs.tofile(os.path.join(d, "bufs.bin"))
            ref = bufs
        O.run_buffers(sched, np.ascontiguousarray(ref), pick_by_worker=(pick == 0))
    text = dict(N=N, W=W, T=T, seed=seed, family=family, mode=mode, source=source, gap_scope=scope,
                n_layers=len(layers) if layers else 0, nesterov=nesterov, track_gap=track_gap, bf16=bf16, n_bufs=n_bufs,
                pick=pick, queue=queue, resident_bytes=resident_bytes, eta=eta, gamma=gamma, sigma=sigma,
                diag_worker=diag_worker, static_diag=static_diag, theta0=int(theta0))
    with open(os.path.join(d, "scenario.txt"), "w") as f:
        for k, v in text.items():
            f.write("%s %r\n" % (k, v))
    r = subprocess.run([driver, d], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0 and "cpu device driver ok" in r.stdout, r.stdout[-4000:]
    raw = np.fromfile(os.path.join(d, "state.bin"), np.uint8)
    pos = [0]

    def take(dtype, count):
        n = np.dtype(dtype).itemsize * count
        x = raw[pos[0]:pos[0] + n].view(dtype)
        pos[0] += n
        return x
    keeps_m = mode in (3, 4) or bool(track_gap)
    got = dict(theta=take(np.float32, N), x=take(np.float32, N))
    if keeps_m:
        got["m"] = take(np.float32, N)
        got["snaps"] = take(np.float32, W * N).reshape(W, N)
    if family == 1:
        got["vw"] = take(np.float32, W * N).reshape(W, N)
    if family == 2:
        got["v2"] = take(np.float32, N)
    got["iter"] = take(np.uint64, W)
    if keeps_m:
        d4 = take(np.float64, 3)
        got["diag"] = dict(mean_graw=d4[0], frac_gt1=d4[1], frac_gt0=d4[2], n_nonfinite=int(take(np.uint64, 1)[0]))
        got["diag_ref"] = O.gap_statistics(diag_worker)
    if scope:
        got["gaps"] = take(np.float32, 1 if scope == 2 else len(layers))
    assert pos[0] == raw.size
    return got, O


def same_bits(a, b):
    return np.array_equal(np.ascontiguousarray(a, np.float32).view(np.uint32), np.ascontiguousarray(b, np.float32).view(np.uint32))


def check(got, O, family=0, exact=True):
    cmp = same_bits if exact else (lambda a, b: np.allclose(a, b, rtol=1e-6, atol=1e-37, equal_nan=True))
    assert cmp(got["theta"], O.theta), "theta"
    assert cmp(got["x"], {0: lambda: O.v, 1: lambda: O.vsum, 2: lambda: O.m1}[family]()), "v / sum of v / m1"
    if "m" in got:
        assert cmp(got["m"], O.m), "m"
        assert cmp(got["snaps"], O.snaps), "snapshots"
    if family == 1:
        assert cmp(got["vw"], O.vw), "worker momenta"
    if family == 2:
        assert cmp(got["v2"], O.v2), "second moment"
    assert np.array_equal(got["iter"], O.iter)
    if "diag" in got:
        d, r = got["diag"], got["diag_ref"]
        N = got["theta"].size
        assert d["n_nonfinite"] == r["n_nonfinite"]
        assert round(d["frac_gt1"] * N) == r["n_gt1"] and round(d["frac_gt0"] * N) == r["n_gt0"]
        assert abs(d["mean_graw"] - r["mean_graw"]) <= 1e-6 * abs(r["mean_graw"]) + 1e-300


# sizes: below one group of four, below one block, several blocks with ragged tails of every residue
SIZES = [1, 3, 67, 1025, 4098, 9001, 20483]


@pytest.mark.parametrize("N", SIZES)
@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4])
def test_fused_update_one_launch_per_arrival(driver, tmp_path, N, mode):
    # gradient buffers of exactly N values (float, then bfloat16), picked by worker; a resident budget that cuts
    # inside theta, v and m so that the launch takes several hint paths
    for bf16 in (0, 1):
        got, O = run(driver, tmp_path, N, 3, 7, 100 + N, mode=mode, source=2, bf16=bf16, track_gap=N % 2,
                     resident_bytes=5 * N, static_diag=1)
        check(got, O)


@pytest.mark.parametrize("N", SIZES)
@pytest.mark.parametrize("family", [0, 1, 2])
def test_persistent_kernel_with_the_quadratic_source(driver, tmp_path, N, family):
    got, O = run(driver, tmp_path, N, 4, 25, 200 + N, family=family, mode=3, source=0, eta=0.01 if family == 2 else 0.1)
    check(got, O, family)
    got, O = run(driver, tmp_path, N, 2, 9, 300 + N, family=family, mode=1, source=0, track_gap=1, eta=0.01 if family == 2 else 0.1)
    check(got, O, family)


@pytest.mark.parametrize("N", [3, 1025, 9001])
@pytest.mark.parametrize("family", [0, 1, 2])
def test_quadratic_source_one_launch_per_arrival_and_queues(driver, tmp_path, N, family):
    eta = 0.01 if family == 2 else 0.1
    got, O = run(driver, tmp_path, N, 3, 8, 400 + N, family=family, mode=4, source=1, eta=eta)
    check(got, O, family)
    # gradient buffers in the persistent kernel, and the second part of the arrivals as a queue
    got, O = run(driver, tmp_path, N, 3, 11, 500 + N, family=family, mode=3, source=3, pick=1, eta=eta)
    check(got, O, family)
    got, O = run(driver, tmp_path, N, 3, 11, 600 + N, family=family, mode=3, source=3, bf16=1, eta=eta)
    check(got, O, family)
    got, O = run(driver, tmp_path, N, 3, 11, 700 + N, family=family, mode=3, source=2, queue=1, eta=eta)
    check(got, O, family)


@pytest.mark.parametrize("family", [0, 1, 2])
def test_start_other_than_zero(driver, tmp_path, family):
    # ga_set_theta scatters theta_0 into the tiled state and copies it to every snapshot
    eta = 0.01 if family == 2 else 0.1
    got, O = run(driver, tmp_path, 20483, 3, 9, 900 + family, family=family, mode=3, source=0, eta=eta, theta0=True)
    check(got, O, family)
    got, O = run(driver, tmp_path, 9001, 3, 9, 910 + family, family=family, mode=3, source=2, eta=eta, theta0=True)
    check(got, O, family)


@pytest.mark.parametrize("nesterov", [0, 1])
def test_nesterov_form(driver, tmp_path, nesterov):
    got, O = run(driver, tmp_path, 4098, 3, 9, 31, mode=3, source=2, nesterov=nesterov)
    check(got, O)
    got, O = run(driver, tmp_path, 4098, 3, 9, 32, mode=3, source=0, nesterov=nesterov)
    check(got, O)


@pytest.mark.parametrize("scope,layers", [(1, [5, 4097, 64, 8300, 1, 700]), (1, [13167]), (2, None)])
@pytest.mark.parametrize("mode", [3, 4])
def test_layer_wise_and_global_gap(driver, tmp_path, scope, layers, mode):
    N = 13167
    for bf16 in (0, 1):
        got, O = run(driver, tmp_path, N, 3, 7, 800 + mode, mode=mode, source=2, scope=scope, layers=layers, bf16=bf16,
                     resident_bytes=6 * N)
        # the layer sums are added in another order than the oracle's: the criterion of the GPU tests
        check(got, O, exact=False)
        assert np.allclose(got["gaps"], O.last_gaps, rtol=1e-6)
