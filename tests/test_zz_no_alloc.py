"""The entry point for callers that cannot allocate: ga_gap_statistics_static keeps its reduction partials in a
static device array of the library.  Checked against ga_diagnostics (the existing entry point with the partials in
the caller's workspace) on two calls in a row, the second with a smaller input that leaves most of the array's
previous contents in place."""
import numpy as np
import pytest
import torch

import ga_inputs
import paper_1909_10802_amd as ga
from gpu_util import dev, load_state

pytestmark = pytest.mark.gpu


def reference(N, W, theta, v, m, snaps, k, w):
    """ga_diagnostics of a context that holds the first N parameters of the state."""
    M = ga.Master(N, W, mode=ga.GA_MODE_GA)
    load_state(M, theta[:N], v[:N], m[:N], snaps[:, :N], k, np.full(W, k, np.uint64))
    d = M.diagnostics(w)
    M.close()
    return d


def test_static_scratch_entry_point_matches_ga_diagnostics():
    W, seed, k = 3, 77, 40
    N1, N2 = 3_000_003, 70_001                       # 2048 partials, then 69 of them
    theta, v, m, snaps = ga_inputs.random_state(N1, W, seed)
    snaps[1, 5] = np.inf
    theta[N2 - 2] = np.nan
    snaps[1, 100:200] = theta[100:200]
    h = ga_inputs.rng(seed, 9)
    big = h.integers(0, N1, size=1000)
    snaps[1, big] += np.float32(10.0)                # some Gaps far above one
    d_theta, d_m, d_snap = dev(theta), dev(m), dev(snaps[1])
    out1 = torch.zeros(ga.DIAG_BYTES, dtype=torch.uint8, device="cuda:0")
    out2 = torch.zeros(ga.DIAG_BYTES, dtype=torch.uint8, device="cuda:0")
    hy = dict(beta=0.999, eta_max=0.1, eps=1e-8)
    ga.ga_gap_statistics_static(d_theta, d_snap, d_m, N1, k, hy["beta"], hy["eta_max"], hy["eps"], out1)
    ga.ga_gap_statistics_static(d_theta, d_snap, d_m, N2, k, hy["beta"], hy["eta_max"], hy["eps"], out2)
    got1, got2 = ga.diag_from_device(out1), ga.diag_from_device(out2)
    for N, got in ((N1, got1), (N2, got2)):
        ref = reference(N, W, theta, v, m, snaps, k, 1)
        assert got["n_nonfinite"] == ref["n_nonfinite"] and got["n_nonfinite"] >= 1
        assert round(got["frac_gt1"] * N) == round(ref["frac_gt1"] * N) > 0
        assert round(got["frac_gt0"] * N) == round(ref["frac_gt0"] * N)
        assert abs(got["mean_graw"] - ref["mean_graw"]) <= 1e-6 * abs(ref["mean_graw"])
        assert got == ref                             # same kernels, same summation order: the same bits


def test_static_scratch_entry_point_rejects_bad_arguments():
    x = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    out = torch.zeros(ga.DIAG_BYTES, dtype=torch.uint8, device="cuda:0")
    L = ga.lib()
    p, o, s = x.data_ptr(), out.data_ptr(), torch.cuda.current_stream().cuda_stream
    assert L.ga_gap_statistics_static(p, p, p, (1 << 40) + 1, 1, 0.999, 0.1, 1e-8, o, s) == ga.GA_ERR_ARG
    assert b"maximum" in L.ga_last_error(None)
    assert L.ga_gap_statistics_static(p, p, p, 0, 1, 0.999, 0.1, 1e-8, o, s) == ga.GA_ERR_ARG
    assert L.ga_gap_statistics_static(None, p, p, 64, 1, 0.999, 0.1, 1e-8, o, s) == ga.GA_ERR_ARG
    assert L.ga_gap_statistics_static(p + 4, p, p, 32, 1, 0.999, 0.1, 1e-8, o, s) == ga.GA_ERR_ALIGN
    assert L.ga_gap_statistics_static(p, p, p, 64, 1, 0.999, 0.1, 0.0, o, s) == ga.GA_ERR_ARG
    torch.cuda.synchronize()
