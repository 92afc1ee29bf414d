"""What the paper reports about the penalties, seen on the HIP path at the full size of
the smallest workload (no oracle involved: these are properties, not parity).

  * App. C.8 / Sec. 4.3: over a run the mean parameter-wise Gap stays well below the mean delay.
  * Sec. 2 and Sec. 5: with momentum and several workers, ASGD without a penalty blows up at a step
    size where the Staleness-Aware and Gap-Aware masters keep descending.
"""
import numpy as np
import pytest
import torch

import ga_inputs
import paper_1909_10802_amd as ga

pytestmark = pytest.mark.gpu


def test_gap_below_delay_and_penalties_stabilise_momentum():
    cfg = ga_inputs.WORKLOADS["cfg1"]
    N, W, T, seed = cfg["N"], cfg["W"], 1600, cfg["seed"]
    chunk = 40
    a, ts = ga_inputs.device_curvatures(N, seed), ga_inputs.device_optimum(N, seed)
    sched = ga.ga_simulate_schedule(W, T + 1, ga.GA_DIST_EXP, 1.0, seed)
    f = lambda th: float(0.5 * (a.double() * (th.double() - ts.double()) ** 2).sum())
    f0 = f(torch.zeros_like(ts))
    loss = {}
    for mode in ("asgd", "sa", "ga"):
        M = ga.Master(N, W, mode=mode, track_gap=True)
        src = ga.quadratic_source(a, ts, seed)
        gaps = []
        for s in range(0, T, chunk):
            M.run_schedule(sched[s:s + chunk], src)
            gaps.append(1.0 + M.diagnostics(int(sched[s + chunk]))["mean_graw"])
        loss[mode] = f(M.theta())
        if mode == "ga":
            mean_tau = float(M.delays()[W:].mean())
            assert abs(mean_tau - W) < 0.05
            assert 1.0 < np.mean(gaps) < 0.5 * mean_tau, (np.mean(gaps), mean_tau)
        M.close()
    assert not loss["asgd"] < f0
    assert loss["sa"] < 1e-2 * f0 and loss["ga"] < 1e-2 * f0, loss
