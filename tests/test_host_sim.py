"""The host side of the library on a CPU: ga_host.cpp is compiled with g++ under AddressSanitizer and
UndefinedBehaviorSanitizer against stand-ins for the HIP runtime and for the kernel launchers (tests/host_sim/), and
driven through every way of delivering arrivals.  What the host decided -- k, iter[], the delays of Alg. 3 / Alg. 5,
and the scalars handed to the kernels for each arrival -- is compared with the oracle's bookkeeping; any sanitizer
report fails the run.  No GPU and no kernel is involved: the arithmetic of the update is the GPU tests' business."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SIM = os.path.join(ROOT, "tests", "host_sim")
CSRC = os.path.join(ROOT, "paper_1909_10802_amd", "csrc")
HIP_INCLUDE = "/opt/rocm/include"
ROW = np.dtype([("worker", np.uint32), ("tau", np.float32), ("lr", np.float32), ("inv_bc_prev", np.float32), ("path", np.int32)])
ETA, BETA = np.float32(0.05), float(np.float32(0.999))
DELAY_LOG = 1 << 20

pytestmark = pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(HIP_INCLUDE),
                                reason="needs g++ and the HIP headers")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host_sim") / "driver")
    subprocess.check_call(["g++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I" + HIP_INCLUDE,
                           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1", "-Wall", "-Wextra",
                           os.path.join(CSRC, "ga_host.cpp"), os.path.join(SIM, "fake_runtime.cpp"),
                           os.path.join(SIM, "fake_launchers.cpp"),
                           os.path.join(SIM, "driver.cpp"), "-o", exe])
    return exe


def run(driver, tmp_path, family, mode, scope, W, T, seed):
    out = str(tmp_path / "host.bin")
    r = subprocess.run([driver, out, str(family), str(mode), str(scope), str(W), str(T), str(seed)],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0 and "host driver ok" in r.stdout, r.stdout[-3000:]
    raw = open(out, "rb").read()
    T_, kept, W_ = np.frombuffer(raw, np.uint64, 3)
    assert (T_, W_) == (T, W)
    o = 24
    sched = np.frombuffer(raw, np.uint32, T, o); o += 4 * T
    it = np.frombuffer(raw, np.uint64, W, o); o += 8 * W
    delays = np.frombuffer(raw, np.uint64, int(kept), o); o += 8 * int(kept)
    rows = np.frombuffer(raw, ROW, T, o)
    assert o + ROW.itemsize * T == len(raw)
    return sched, it, delays, rows


# family, mode, gap scope: momentum in all five modes, DANA and Adam in theirs, layer-wise and global Gap
SCENARIOS = [(0, 0, 0), (0, 1, 0), (0, 2, 0), (0, 3, 0), (0, 4, 0), (1, 0, 0), (1, 1, 0), (1, 3, 0), (2, 1, 0), (2, 4, 0),
             (0, 3, 1), (0, 4, 2)]


@pytest.mark.parametrize("family,mode,scope", SCENARIOS)
@pytest.mark.parametrize("W,T,seed", [(1, 37, 1), (5, 4000, 11), (32, 40003, 2)])   # the last: more than one arrival table (8192 rows) per call
def test_host_bookkeeping_and_scalars(driver, tmp_path, family, mode, scope, W, T, seed):
    sched, it, delays, rows = run(driver, tmp_path, family, mode, scope, W, T, seed)
    assert np.array_equal(sched, oracle.simulate_schedule(W, T, oracle.DIST_EXP, 1.0, seed))
    taus, it_ref = oracle.delays(W, sched)
    assert np.array_equal(it, it_ref) and np.array_equal(delays, taus)
    assert np.array_equal(rows["worker"], sched)
    assert np.array_equal(rows["tau"], taus.astype(np.float32))
    # Alg. 14's bias correction as the kernels receive it: (float)(1 / (1 - beta^(k-1))), 0 at the first arrival
    k = np.arange(1, T + 1, dtype=np.float64)
    want = np.zeros(T, np.float32)
    want[1:] = (1.0 / (1.0 - np.power(BETA, k[1:] - 1.0))).astype(np.float32)
    assert np.array_equal(rows["inv_bc_prev"], want)
    # step size: eta, in the third quarter of the arrivals the per-arrival eta_k; divided by the delay in Alg. 3's form
    part = T // 4
    eta_k = np.full(T, ETA, np.float32)
    i = np.arange(part)
    eta_k[2 * part:3 * part] = ETA * (np.float32(1.0) + (i % 7).astype(np.float32) / np.float32(8.0))
    lr = eta_k / rows["tau"] if mode == 2 else eta_k
    assert np.array_equal(rows["lr"], lr.astype(np.float32))
    # which launcher saw which arrival
    one = {0: 0, 1: 3, 2: 4}[family] if scope == 0 else 5
    path = np.full(T, one, np.int32)
    if scope == 0:
        path[:part] = 1
        path[3 * part:] = 2
    assert np.array_equal(rows["path"], path)


def test_delay_log_wraps(driver, tmp_path):
    W, T, seed = 3, DELAY_LOG + 5000, 7
    sched, it, delays, rows = run(driver, tmp_path, 0, 3, 0, W, T, seed)
    taus, it_ref = oracle.delays(W, sched)
    assert delays.size == DELAY_LOG and np.array_equal(delays, taus[-DELAY_LOG:])
    assert np.array_equal(it, it_ref) and np.array_equal(rows["tau"], taus.astype(np.float32))
