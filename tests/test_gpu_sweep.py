"""GPU-vs-oracle parity across the switch between the two persistent-kernel widths and over a
seeded random sweep of sizes, worker counts, families, penalties and gradient sources (needs an MI355X)."""
import numpy as np
import pytest
import torch

import ga_inputs
import oracle
import paper_1909_10802_amd as ga
from gpu_util import DEV, bits_equal, dev, host
from test_gpu_families import compare as compare_family, make_pair

pytestmark = pytest.mark.gpu

WIDE = 1 << 21          # from this many parameters on the persistent kernel keeps four per thread instead of two


def check_momentum(M, O, what, keep_m):
    torch.cuda.synchronize()
    th = host(M.theta())
    assert bits_equal(th, O.theta) == 0, what + " theta"
    assert bits_equal(host(M.v()), O.v) == 0, what + " v"
    if keep_m:
        assert bits_equal(host(M.m()), O.m) == 0, what + " m"
        for w in range(M.W):
            assert bits_equal(host(M.snapshot(w)), O.snaps[w]) == 0, what + " snapshot %d" % w
    assert M.k == O.k and np.array_equal(M.iter(), O.iter)
    assert np.array_equal(M.delays(), np.array(O.tau_log, np.uint64))


@pytest.mark.parametrize("N", [WIDE - 1, WIDE, WIDE + 3])
@pytest.mark.parametrize("family", [ga.GA_FAMILY_MOMENTUM, ga.GA_FAMILY_DANA, ga.GA_FAMILY_ADAM], ids=["momentum", "dana", "adam"])
def test_persistent_width_switch_full_vector(N, family):
    W, T, seed = 3, 14, 21
    a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
    sched = np.array([0, 1, 2, 2, 0, 1, 1, 0, 2, 0, 0, 1, 2, 1], dtype=np.uint32)
    src = ga.quadratic_source(dev(a), dev(ts), seed)
    if family == ga.GA_FAMILY_MOMENTUM:
        M = ga.Master(N, W, mode=ga.GA_MODE_GA)
        O = oracle.Master(N, W, oracle.MODE_GA, oracle.Hyper())
        M.run_schedule(sched, src)
        O.run_quadratic(sched, a, ts, seed)
        check_momentum(M, O, "width switch N=%d" % N, True)
    else:
        M, O = make_pair(family, N, W, ga.GA_MODE_GA, 0.1 if family == ga.GA_FAMILY_DANA else 0.01, track=False)
        M.run_schedule(sched, src)
        O.run_quadratic(sched, a, ts, seed)
        compare_family(M, O, "width switch N=%d" % N)
    M.close()


def _cases(n, seed):
    r = np.random.default_rng(seed)
    out = []
    for c in range(n):
        N = int(r.choice([r.integers(1, 70), r.integers(70, 5000), r.integers(5000, 150_000)]))
        W = int(r.integers(1, 13))
        T = int(r.integers(1, 70))
        family = int(r.integers(0, 3))
        mode = int(r.choice([0, 1, 3, 4] if family else [0, 1, 2, 3, 4]))
        source = str(r.choice(["persistent", "per_arrival", "f32", "bf16"]))
        nesterov = bool(family == 0 and r.integers(0, 3) == 0)
        dist = int(r.integers(0, 3))
        # cache-resident budget: the default, none, or a cut somewhere inside theta, v, m (so that one launch takes
        # several of the hint paths of the fused update)
        budget = int(r.choice([240 << 20, 0, int(r.integers(0, 12 * N + 1))]))
        out.append((c, N, W, T, family, mode, source, nesterov, dist, budget))
    return out


@pytest.mark.parametrize("case", _cases(192, 20260), ids=lambda c: "c%d-N%d-W%d-T%d-f%d-m%d-%s%s-d%d-b%d" % (c[:7] + ("-nag" if c[7] else "", c[8], c[9])))
def test_random_sweep(case):
    c, N, W, T, family, mode, source, nesterov, dist, budget = case
    seed = 1000 + c
    eta = 0.01 if family == ga.GA_FAMILY_ADAM else 0.1
    sched = ga.ga_simulate_schedule(W, T, dist, 0.7, seed)
    assert np.array_equal(sched, oracle.simulate_schedule(W, T, dist, 0.7, seed))
    track = bool(c % 2)
    if family == ga.GA_FAMILY_MOMENTUM:
        M = ga.Master(N, W, eta=eta, mode=mode, track_gap=track, nesterov=nesterov)
        O = oracle.Master(N, W, mode, oracle.Hyper(eta, 0.9), track_gap=track, nesterov=nesterov)
    else:
        M, O = make_pair(family, N, W, mode, eta, track=track)
    ga.ga_set_resident_bytes(M.ctx, budget)
    if source in ("persistent", "per_arrival"):
        a, ts = ga_inputs.curvatures(N, seed), ga_inputs.optimum(N, seed)
        scratch = torch.empty(N, dtype=torch.float32, device=DEV)
        src = ga.quadratic_source(dev(a), dev(ts), seed, 0.02, source == "persistent", scratch)
        cut = T // 3
        M.run_schedule(sched[:cut], src)
        M.run_schedule(sched[cut:], src)
        O.run_quadratic(sched, a, ts, seed, sigma=0.02)
    else:
        n_bufs = 1 + c % 4
        bufs = ga_inputs.gradient_buffers(n_bufs, N, seed=seed, std=0.3)
        if source == "bf16":
            bits = ga_inputs.f32_to_bf16_bits(bufs).reshape(n_bufs, N)
            ref, dbufs = oracle.bf16_to_f32(bits).reshape(n_bufs, N), [dev(b.view(np.int16)).view(torch.bfloat16) for b in bits]
        else:
            ref, dbufs = bufs, [dev(b) for b in bufs]
        pick = ga.GA_PICK_BY_WORKER if c % 3 else ga.GA_PICK_BY_ARRIVAL
        M.run_schedule(sched, ga.buffer_source(dbufs, pick))
        O.run_buffers(sched, np.ascontiguousarray(ref), pick_by_worker=(pick == ga.GA_PICK_BY_WORKER))
    keep_m = track or mode in (3, 4)
    if family == ga.GA_FAMILY_MOMENTUM:
        check_momentum(M, O, "case %d" % c, keep_m)
    else:
        compare_family(M, O, "case %d" % c, keep_m=keep_m, snaps=keep_m)
    M.close()
