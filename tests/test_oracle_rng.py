"""Pins for the oracle's generators (no GPU)."""
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l[0] not in "#\n"]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]


def test_philox_counter_and_key_sensitivity():
    base = oracle.philox4x32_10([1, 2, 3, 4], [5, 6])
    for pos in range(4):
        c = [1, 2, 3, 4]
        c[pos] ^= 1
        assert not np.array_equal(oracle.philox4x32_10(c, [5, 6]), base)
    assert not np.array_equal(oracle.philox4x32_10([1, 2, 3, 4], [5, 7]), base)
    assert not np.array_equal(oracle.philox4x32_10([1, 2, 3, 4], [4, 6]), base)


def test_noise_matches_box_muller_in_double():
    # The float transform (Taylor series, float rounding) against the Box-Muller
    # definition evaluated with libm in double on the same random bits.
    worst = 0.0
    for seed, k in [(1, 1), (2, 77), (2**40 + 3, 2**33 + 5)]:
        z = oracle.noise_f32(seed, k, 0, 1 << 19).astype(np.float64)
        r = oracle.noise_ref(seed, k, 0, 1 << 19)
        worst = max(worst, np.abs(z - r).max())
        assert np.all(np.abs(z - r) <= 1.5e-6 * np.maximum(1.0, np.abs(r)))
    assert worst > 0.0      # it is a float approximation, not the same routine


def test_noise_moments():
    n = 1 << 22
    z = oracle.noise_f32(12345, 9, 0, n).astype(np.float64)
    assert abs(z.mean()) < 5 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 5 * np.sqrt(2.0 / n)
    assert abs((z ** 3).mean()) < 5 * np.sqrt(15.0 / n)
    assert abs((z ** 4).mean() - 3.0) < 5 * np.sqrt(96.0 / n)
    # standard normal quantiles
    for q, x in [(0.5, 0.0), (0.8413447, 1.0), (0.9772499, 2.0), (0.0013499, -3.0)]:
        assert abs((z < x).mean() - q) < 5 * np.sqrt(q * (1 - q) / n)
    # neighbours in j (same Philox block, other lane / other pair / next block)
    for lag in (1, 2, 3, 4):
        c = (z[:-lag] * z[lag:]).mean()
        assert abs(c) < 5 / np.sqrt(n), (lag, c)
    # sine and cosine of one pair share the radius but are uncorrelated, and
    # their squares sum to r^2 ~ chi-square(2): mean 2, variance 4
    r2 = z[0::2] ** 2 + z[1::2] ** 2
    assert abs(r2.mean() - 2.0) < 5 * np.sqrt(4.0 / (n / 2))
    assert abs(r2.var() - 4.0) < 0.05


def test_noise_independent_across_arrivals_and_seeds():
    n = 1 << 20
    z1 = oracle.noise_f32(7, 1, 0, n).astype(np.float64)
    z2 = oracle.noise_f32(7, 2, 0, n).astype(np.float64)
    z3 = oracle.noise_f32(8, 1, 0, n).astype(np.float64)
    assert abs((z1 * z2).mean()) < 5 / np.sqrt(n)
    assert abs((z1 * z3).mean()) < 5 / np.sqrt(n)


def test_noise_is_a_function_of_the_global_index():
    # z(seed, k, j) must not depend on where the evaluation window starts.
    full = oracle.noise_f32(3, 11, 0, 4096)
    for j0 in (1, 2, 3, 5, 1023):
        part = oracle.noise_f32(3, 11, j0, 64)
        assert np.array_equal(part, full[j0:j0 + 64])
    far = 2**34 + 6
    assert np.array_equal(oracle.noise_f32(3, 11, far, 8)[2:], oracle.noise_f32(3, 11, far + 2, 6))
    assert np.all(np.isfinite(oracle.noise_f32(3, 11, far, 1024)))


def test_noise_range():
    z = oracle.noise_f32(99, 3, 0, 1 << 22)
    assert np.all(np.isfinite(z))
    assert np.abs(z).max() <= np.sqrt(2 * 24 * np.log(2.0)) + 1e-5   # u1 >= 2^-24
