"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

import oracle
import paper_1909_10802_amd as ga

DEV = "cuda:0"
MODES = [ga.GA_MODE_ASGD, ga.GA_MODE_SA, ga.GA_MODE_SA_STEP, ga.GA_MODE_GA, ga.GA_MODE_GA_HINGE]
MODE_NAMES = {v: k for k, v in ga.MODES.items()}

# Per-step tolerance: relative 1e-6 on every state element (float).  The kernels
# perform the same correctly rounded float operations in the same order as the
# oracle, so the observed difference is zero; the absolute floor only admits
# differences below the smallest normal float.
RTOL_STEP = 1e-6
ATOL_STEP = 1e-37
# Whole trajectory: relative L2 error of theta.
RTOL_TRAJ_L2 = 1e-5


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def bits_equal(a, b):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    return int(np.count_nonzero(a.view(np.uint32) != b.view(np.uint32)))


def assert_step_close(got, ref, what):
    got, ref = np.asarray(got, dtype=np.float32), np.asarray(ref, dtype=np.float32)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    both_nan = np.isnan(got) & np.isnan(ref)
    same_inf = np.isinf(ref) & (got == ref)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    ok = (err <= RTOL_STEP * np.abs(ref.astype(np.float64)) + ATOL_STEP) | both_nan | same_inf
    if not ok.all():
        j = int(np.argmin(ok))
        raise AssertionError("%s: %d of %d elements differ; first at %d: gpu %r oracle %r"
                             % (what, (~ok).sum(), ok.size, j, got.flat[j], ref.flat[j]))


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    d = np.linalg.norm(np.asarray(got, dtype=np.float64) - ref)
    n = np.linalg.norm(ref)
    return d / n if n > 0 else d


def load_state(M, theta, v, m, snaps, k=0, it=None):
    """Put a given state into a GPU master (teacher forcing)."""
    ga.ga_put_theta(M.ctx, dev(theta))
    ga.ga_put_v(M.ctx, dev(v))
    ga.ga_put_m(M.ctx, dev(m))
    for w in range(M.W):
        ga.ga_put_snapshot(M.ctx, w, dev(snaps[w]))
    ga.ga_set_bookkeeping(M.ctx, k, np.zeros(M.W, np.uint64) if it is None else it)


def gpu_state(M):
    torch.cuda.synchronize()
    return (host(M.theta()), host(M.v()), host(M.m()), np.stack([host(M.snapshot(w)) for w in range(M.W)]))


def compare_masters(M, O, what, snaps=True, keep_m=True, exact=True):
    th, v, m, sn = gpu_state(M)
    assert_step_close(th, O.theta, what + " theta")
    assert_step_close(v, O.v, what + " v")
    if keep_m:
        assert_step_close(m, O.m, what + " m")
    if snaps:
        assert_step_close(sn, O.snaps, what + " snapshots")
    assert M.k == O.k, what
    assert np.array_equal(M.iter(), O.iter), what
    assert np.array_equal(M.delays(), np.array(O.tau_log, np.uint64)), what
    if exact:
        assert bits_equal(th, O.theta) == 0 and bits_equal(v, O.v) == 0, what + ": not bit-identical"


def oracle_hyper(eta=0.1, gamma=0.9, **kw):
    return oracle.Hyper(eta, gamma, **kw)
