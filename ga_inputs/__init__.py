"""Seeded synthetic inputs for the Gap-Aware master update.

Shared by the tests, the benchmark and the smoke check to feed BOTH the CPU
oracle and the GPU library with the same data.  It contains none of the
method's arithmetic: only random draws with numpy's generators and the sizes
of the five workloads.

The workloads stand in for the paper's experiments (Sec. 6, App. C.2/C.4):
only the model sizes and worker counts are taken from them; the loss is a
separable quadratic with curvatures a ~ U[0.1, 1) and optimum theta* ~ N(0,1),
or precomputed Gaussian gradient buffers.
"""
import numpy as np

# name -> workload description
WORKLOADS = {
    # ResNet-20-sized
    "cfg1": dict(N=272_474, W=8, T=1_000, dist="exp", sigma=1.0, source="quadratic", seed=1,
                 grad_dtype="f32", eta=0.1, gamma=0.9),
    # WRN-16-4-sized
    "cfg2": dict(N=2_748_890, W=32, T=10_000, dist="exp", sigma=1.0, source="quadratic", seed=2,
                 grad_dtype="f32", eta=0.1, gamma=0.9),
    # ResNet-50-sized, 161 tensors, one gradient buffer per worker
    "cfg3": dict(N=25_557_032, W=64, T=2_000, dist="exp", sigma=1.0, source="buffers", n_bufs=64,
                 pick="worker", n_tensors=161, seed=3, grad_dtype="f32", grad_std=1e-2, eta=0.1, gamma=0.9),
    # Transformer-XL-base-sized, heavy-tailed iteration times
    "cfg4": dict(N=151_000_000, W=128, T=5_000, dist="lognormal", sigma=1.0, source="quadratic", seed=4,
                 grad_dtype="f32", eta=0.1, gamma=0.9),
    # capacity stress: bf16 gradients, 128 fp32 snapshots
    "cfg5": dict(N=350_000_000, W=128, T=1_000, dist="hetero", sigma=1.5, source="buffers", n_bufs=4,
                 pick="arrival", seed=5, grad_dtype="bf16", grad_std=1e-2, eta=0.1, gamma=0.9),
}

DIST_CODES = {"exp": 0, "lognormal": 1, "hetero": 2}


def rng(seed, stream):
    """Independent numpy generator for (seed, stream)."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def curvatures(N, seed, lo=0.1, hi=1.0):
    """a ~ U[lo, hi), float32."""
    return (lo + (hi - lo) * rng(seed, 1).random(N, dtype=np.float32)).astype(np.float32)


def optimum(N, seed):
    """theta* ~ N(0, 1), float32."""
    return rng(seed, 2).standard_normal(N, dtype=np.float32)


def gradient_buffers(n_bufs, N, seed, std=1e-2):
    """n_bufs rows of N(0, std) float32 gradients."""
    out = rng(seed, 3).standard_normal((n_bufs, N), dtype=np.float32)
    out *= np.float32(std)
    return out


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def tensor_sizes(N, n_tensors, seed, min_size=64):
    """Random composition of N into n_tensors contiguous tensors, each >= min_size."""
    assert N >= n_tensors * min_size
    free = N - n_tensors * min_size
    cuts = np.sort(rng(seed, 4).integers(0, free + 1, size=n_tensors - 1))
    parts = np.diff(np.concatenate(([0], cuts, [free]))) + min_size
    assert parts.sum() == N and parts.min() >= min_size
    return parts.astype(np.uint64)


def random_state(N, W, seed, scale=1.0):
    """A generic mid-trajectory state for single-step checks: theta, v, m >= 0, W snapshots."""
    g = rng(seed, 5)
    theta = (scale * g.standard_normal(N)).astype(np.float32)
    v = (0.1 * scale * g.standard_normal(N)).astype(np.float32)
    m = ((0.1 * scale) ** 2 * g.random(N)).astype(np.float32)
    snaps = (theta[None, :] + 0.05 * scale * g.standard_normal((W, N))).astype(np.float32)
    return theta, v, m, snaps


def sample_indices(N, n_random, seed, boundaries=()):
    """Index set for sampled parity on very large vectors: head, tail, tensor
    boundaries +-8 and n_random seeded indices; sorted and unique."""
    parts = [np.arange(min(4096, N)), np.arange(max(0, N - 4096), N)]
    for b in boundaries:
        parts.append(np.arange(max(0, int(b) - 8), min(N, int(b) + 8)))
    parts.append(rng(seed, 6).integers(0, N, size=n_random))
    return np.unique(np.concatenate(parts)).astype(np.uint64)


# ---------------------------------------------------------------- device-side generators
# For the full-size workloads the inputs are drawn on the GPU with torch's
# seeded generator (drawing 10^8..10^9 normals with numpy would dominate the
# run).  They are inputs like the numpy ones above: the oracle gets the same
# values copied back (whole, or gathered at the sampled indices).
def device_generator(seed, stream, device="cuda:0"):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + int(stream))
    return g


def device_curvatures(N, seed, device="cuda:0", lo=0.1, hi=1.0):
    import torch
    u = torch.rand(N, dtype=torch.float32, device=device, generator=device_generator(seed, 1, device))
    return u.mul_(hi - lo).add_(lo)


def device_optimum(N, seed, device="cuda:0"):
    import torch
    return torch.randn(N, dtype=torch.float32, device=device, generator=device_generator(seed, 2, device))


def device_gradient_buffers(n_bufs, N, seed, std=1e-2, dtype="f32", device="cuda:0"):
    """List of n_bufs device tensors of N(0, std) gradients, float32 or bfloat16."""
    import torch
    g = device_generator(seed, 3, device)
    out = []
    for _ in range(n_bufs):
        x = torch.randn(N, dtype=torch.float32, device=device, generator=g).mul_(std)
        out.append(x.to(torch.bfloat16) if dtype == "bf16" else x)
    return out


def device_gap_state(N, seed, device="cuda:0"):
    """(theta, snapshot, m) as device tensors for a full-size check of the Gap statistics: snapshot = theta plus a small
    normal offset, every fifth parameter unmoved (Gap exactly zero), m uniform in [0, 1e-4), and a few planted
    non-finite and extreme entries at fixed places."""
    import torch
    g = device_generator(seed, 6, device)
    theta = torch.randn(N, dtype=torch.float32, device=device, generator=g)
    snap = torch.randn(N, dtype=torch.float32, device=device, generator=g).mul_(0.002).add_(theta)
    snap[::5] = theta[::5]
    m = torch.rand(N, dtype=torch.float32, device=device, generator=g).mul_(1e-4)
    m[12345] = float("nan")
    snap[N - 2] = float("inf")
    m[7] = float("inf")              # C infinite: Gap 0, finite
    m[N // 2] = 0.0                  # C at its floor eta_max * eps: a huge Gap
    theta[N // 3] = float("nan")
    return theta, snap, m
