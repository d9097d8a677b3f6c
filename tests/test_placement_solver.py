"""Table assignment (Section 5.6.1, Eq. 6): the library's solver (a host function of the
C ABI, no GPU needed) against the enumeration oracle.  CPU only."""
import math

import numpy as np
import pytest

from oracle import placement_oracle as po

RNG = np.random.default_rng


def solve(size, traffic, capacity, bandwidth):
    from paper_2305_01515_amd import placement
    return placement.plan(size, traffic, capacity, bandwidth)


@pytest.mark.parametrize("seed", range(40))
def test_solver_matches_enumeration(seed):
    g = RNG(1000 + seed)
    T = int(g.integers(1, 9))
    Mn = int(g.integers(1, 4))
    size = g.integers(1, 50, size=T).tolist()
    traffic = (g.random(T) ** 3 * 1000).tolist()
    capacity = [int(sum(size) * g.uniform(0.1, 0.8)) for _ in range(Mn)]
    if seed % 3 == 0:
        capacity[-1] = sum(size)
    bandwidth = sorted((g.random(Mn) * 10 + 0.01).tolist(), reverse=seed % 2 == 0)
    ref_a, ref_t = po.best_assignment(size, traffic, capacity, bandwidth)
    res = solve(size, traffic, capacity, bandwidth)
    if ref_a is None:
        assert res is None
        return
    assign, t, optimal = res
    assert optimal
    assert po.feasible(assign, size, capacity)
    assert t == pytest.approx(ref_t, rel=1e-12)
    assert po.lookup_time(assign, traffic, bandwidth) == pytest.approx(ref_t, rel=1e-12)


def test_solver_on_a_hundred_tables_is_feasible_and_not_worse_than_greedy():
    g = RNG(5)
    T = 100
    size = (np.exp(g.uniform(math.log(1e4), math.log(5e7), T)) * 256).astype(np.int64).tolist()
    traffic = (np.exp(g.uniform(0, math.log(100), T)) * 256 * 16384).tolist()
    capacity = [16 << 30, sum(size)]
    bandwidth = [4e12, 45e9]
    assign, t, _ = solve(size, traffic, capacity, bandwidth)
    assert po.feasible(assign, size, capacity)
    # greedy by traffic per byte
    left, greedy = capacity[0], 0.0
    for i in sorted(range(T), key=lambda i: -traffic[i] / size[i]):
        if size[i] <= left:
            left -= size[i]
            greedy += traffic[i] / bandwidth[0]
        else:
            greedy += traffic[i] / bandwidth[1]
    assert t <= greedy * (1 + 1e-12)


def test_solver_errors():
    from paper_2305_01515_amd import placement
    with pytest.raises(ValueError):
        placement.plan([1], [1.0], [], [])
    with pytest.raises(ValueError):
        placement.plan([1, 2], [1.0], [5], [1.0])
    with pytest.raises(ValueError):
        placement.plan([1], [1.0], [5], [0.0])
    with pytest.raises(ValueError):
        placement.plan([-1], [1.0], [5], [1.0])
