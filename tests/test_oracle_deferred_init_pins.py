"""Pins of the oracle's deferred initialisation on read (Section 5.4.2) against things other
than itself: the published first outputs of splitmix64 for the hash, an independent
re-computation of the generator with Python integers, the moments of the twelve-uniform
approximation of a normal distribution, and the property that defines the feature -- training with deferred
initialisation equals training on a table initialised in advance with the same generator,
whatever the order of the reads.  CPU only."""
import math

import numpy as np
import pytest

from oracle import Oracle, lib
from test_oracle_pins import RNG, random_batch

M64 = (1 << 64) - 1


def splitmix_step(x):
    x = (x + 0x9E3779B97F4A7C15) & M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & M64
    return x ^ (x >> 31)


def test_hash_is_splitmix64():
    # first outputs of splitmix64 seeded with 0, as published with its reference implementation
    assert splitmix_step(0) == 0xE220A8397B1DCDAF
    assert splitmix_step(0x9E3779B97F4A7C15) == 0x6E789E6AA1B965F4


def py_sum(seed, t, r, d):
    """centred sum of twelve 16-bit uniforms, all in Python integers"""
    key = splitmix_step(seed ^ (((t + 1) * 0xD1342543DE82EF95) & M64))
    s = -12 * 65536
    for j in range(3):
        h = splitmix_step((key + r * 0x2545F4914F6CDD1D + d * 3 + j) & M64)
        for f in range(4):
            s += 2 * ((h >> (16 * f)) & 0xFFFF) + 1
    return s


def test_generator_matches_python_integers():
    g = RNG(0)
    for _ in range(2000):
        seed, t, r, d = int(g.integers(0, 2 ** 63)), int(g.integers(0, 200)), int(g.integers(0, 2 ** 31)), int(g.integers(0, 512))
        s = py_sum(seed, t, r, d)
        assert lib().orc_init_sum(seed, t, r, d) == s
        std = float(np.float32(g.random() + 0.01))
        # one fp32 product: float(S) * (std * 2^-17); numpy's float32 arithmetic is the reference
        ref = np.float32(s) * np.float32(np.float32(std) * np.float32(2.0 ** -17))
        assert np.float32(lib().orc_init_value(seed, std, t, r, d)) == ref


def test_generator_is_close_to_standard_normal():
    n = 200000
    z = np.array([lib().orc_init_sum(12345, 3, r, d) for r in range(n // 8) for d in range(8)]) / 2.0 ** 17
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 4 * math.sqrt(2.0 / n)
    # twelve uniforms: fourth moment 3 - 1/10 (kurtosis of the Irwin-Hall sum), third moment 0, |z| < 6
    assert abs((z ** 4).mean() - 2.9) < 0.1 and abs((z ** 3).mean()) < 0.05
    assert np.abs(z).max() < 6.0
    assert 0.66 < (np.abs(z) < 1.0).mean() < 0.70 and 0.94 < (np.abs(z) < 2.0).mean() < 0.965
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 0.01                  # neighbouring elements
    assert abs(np.corrcoef(z[:-8], z[8:])[0, 1]) < 0.01                     # neighbouring rows
    other = np.array([lib().orc_init_sum(12345, 4, r, d) for r in range(1000) for d in range(8)]) / 2.0 ** 17
    assert abs(np.corrcoef(z[:8000], other)[0, 1]) < 0.05                   # neighbouring tables


def pre_initialised(rows, dims, dts, seed, std):
    return [np.array([[lib().orc_init_value(seed, std, t, r, d) for d in range(D)] for r in range(H)]).astype(dt)
            for t, (H, D, dt) in enumerate(zip(rows, dims, dts))]


@pytest.mark.parametrize("slots,slots2", [([16, 8], None), ([4, 0], None), ([8, 8], [16, 32])])
def test_deferred_equals_initialised_in_advance(slots, slots2):
    rows, dims, dts, seed, std = [120, 40], [8, 4], [np.float32, np.float16], 77, 0.05
    Wa = pre_initialised(rows, dims, dts, seed, std)
    Ma = [np.zeros(r, dtype=np.float32) for r in rows]
    Wb = [np.full((r, d), np.nan, dtype=dt) for r, d, dt in zip(rows, dims, dts)]  # no value may ever be read
    Mb = [np.zeros(r, dtype=np.float32) for r in rows]
    a = Oracle(Wa, Ma, slots, ways=4, second_level_slots=slots2)
    b = Oracle(Wb, Mb, slots, ways=4, second_level_slots=slots2, deferred_init=(seed, std))
    touched = [set(), set()]
    for k in range(12):
        idx, off = random_batch(rows, 6, 4, seed=500 + k)
        go = RNG(k).standard_normal((6, sum(dims))).astype(np.float32)
        for o in (a, b):
            o.prefetch(idx, off)
        oa, ob = a.forward(), b.forward()
        assert np.array_equal(oa, ob) and np.isfinite(ob).all()
        for o in (a, b):
            o.backward_update(go, 0.05, 1e-8)
        B = 6
        for t in range(2):
            touched[t] |= set(idx[off[t * B]:off[(t + 1) * B]].tolist())
        assert a.stats()[0] == b.stats()[0]
    a.flush()
    b.flush()
    for t in range(2):
        rows_t = sorted(touched[t])
        init = b.initialised(t)
        assert set(np.nonzero(init)[0].tolist()) == touched[t]
        assert np.array_equal(Wa[t][rows_t], Wb[t][rows_t]) and np.array_equal(Ma[t], Mb[t])
        untouched = [r for r in range(rows[t]) if r not in touched[t]]
        assert np.isnan(Wb[t][untouched].astype(np.float64)).all()   # never written


def test_values_do_not_depend_on_the_order_of_first_reads():
    rows, dims, seed, std = [64], [4], 5, 1.0
    res = []
    for order in ([3, 9, 27], [27, 3, 9]):
        W = [np.full((64, 4), np.nan, dtype=np.float32)]
        o = Oracle(W, [np.zeros(64, dtype=np.float32)], [0], ways=2, deferred_init=(seed, std))
        for r in order:
            o.prefetch(np.array([r]), np.array([0, 1]))
            o.forward()
            o.backward_update(np.zeros((1, 4), dtype=np.float32), 0.1, 1e-8)
        res.append(W[0][[3, 9, 27]].copy())
    assert np.array_equal(res[0], res[1])
    assert np.array_equal(res[0][0], np.array([py_sum(5, 0, 3, d) for d in range(4)], dtype=np.float32) * np.float32(2.0 ** -17))


def test_deferred_init_is_fixed_before_the_first_batch():
    W, M = [np.zeros((10, 4), dtype=np.float32)], [np.zeros(10, dtype=np.float32)]
    o = Oracle(W, M, [4], ways=2)
    assert lib().orc_enable_deferred_init(o.h, 1, -1.0) != 0
    o.prefetch(np.array([1]), np.array([0, 1]))
    assert lib().orc_enable_deferred_init(o.h, 1, 1.0) != 0
