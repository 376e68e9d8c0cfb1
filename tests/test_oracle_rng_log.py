"""Pins for the oracle's random numbers and its specified log2 (CPU only)."""
import math
import os

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers(oracle_mod):
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for w in rows:
        v = [int(t, 16) for t in w]
        out = oracle_mod.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def test_uniform_is_open_interval_and_exact(oracle_mod):
    us = np.array([oracle_mod.uniform(3, t, j) for t in range(20) for j in range(500)], np.float64)
    assert us.min() >= 2.0 ** -24 and us.max() <= 1.0 - 2.0 ** -24
    # every value is an odd multiple of 2^-24
    k = us * 2.0 ** 24
    assert np.all(k == np.round(k)) and np.all(k.astype(np.int64) % 2 == 1)


def test_uniform_counter_words(oracle_mod):
    # the draw for (seed, t, j) uses counter (j_lo, j_hi, t_lo, t_hi) and key (seed_lo, seed_hi)
    seed, t, j = 0x1234567890ABCDEF, 0x1_0000_0007, 0x2_0000_0005
    out = oracle_mod.philox4x32_10([j & 0xFFFFFFFF, j >> 32, t & 0xFFFFFFFF, t >> 32],
                                   [seed & 0xFFFFFFFF, seed >> 32])
    m = int(out[0]) >> 9
    assert oracle_mod.uniform(seed, t, j) == (2 * m + 1) * 2.0 ** -24


def test_uniform_is_uniform_chi_square(oracle_mod):
    n, bins = 200000, 64
    us = np.array([oracle_mod.uniform(11, 5, j) for j in range(n)])
    cnt = np.bincount((us * bins).astype(int), minlength=bins)
    chi2 = ((cnt - n / bins) ** 2 / (n / bins)).sum()
    # 63 dof: mean 63, sd 11.2; 140 is beyond the 1e-7 tail
    assert chi2 < 140.0
    # neighbouring counters are uncorrelated
    a, b = us[:-1] - 0.5, us[1:] - 0.5
    assert abs((a * b).mean() / a.var()) < 0.01
    # different round, different seed -> different streams
    assert oracle_mod.uniform(11, 6, 0) != oracle_mod.uniform(11, 5, 0)
    assert oracle_mod.uniform(12, 5, 0) != oracle_mod.uniform(11, 5, 0)


def test_log2_spec_matches_libm(oracle_mod):
    rng = np.random.default_rng(0)
    xs = np.concatenate([
        np.exp2(rng.uniform(-40, 45, 20000)),
        1.0 + rng.uniform(-0.3, 0.45, 5000),                 # the whole reduced interval
        [1.0, 2.0, 0.5, 2.0 ** -24, 1 - 2.0 ** -24, 1 + 2.0 ** -23, 1e-6, 1e12 + 1e-6, 24.0,
         math.sqrt(2.0), np.nextafter(np.float32(math.sqrt(2.0)), np.float32(2.0))],
    ]).astype(np.float32)
    worst = 0.0
    for x in xs:
        ref = math.log2(float(x))
        got = oracle_mod.log2_spec(float(x))
        tol = 3e-7 * max(1.0, abs(ref)) if abs(ref) > 1e-3 else 3e-7 * abs(ref) + 1e-12
        assert abs(got - ref) <= tol, (float(x), got, ref)
        worst = max(worst, abs(got - ref) / max(abs(ref), 1e-30))
    assert oracle_mod.log2_spec(1.0) == 0.0
    assert oracle_mod.log2_spec(8.0) == 3.0
    assert oracle_mod.log2_spec(0.25) == -2.0


def test_log2_spec_monotone_near_one(oracle_mod):
    # relative accuracy just below 1 (u -> 1 gives the largest Gumbel keys)
    for k in (1, 3, 5, 101, 4097):
        x = 1.0 - k * 2.0 ** -24
        ref = math.log2(x)
        assert abs(oracle_mod.log2_spec(x) - ref) <= 2e-7 * abs(ref)
