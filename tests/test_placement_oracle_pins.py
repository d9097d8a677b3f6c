"""Table assignment (Section 5.6.1, Eq. 6): pins of the enumeration oracle against a
textbook 0/1 knapsack, closed forms and a hand-worked case.  CPU only."""
import math

import numpy as np
import pytest

from oracle import placement_oracle as po

RNG = np.random.default_rng


# ---------------------------------------------------------------- oracle pins

def knapsack_max_value(weights, values, cap):
    """textbook dynamic programme over integer capacities"""
    best = [0.0] * (cap + 1)
    for w, v in zip(weights, values):
        for c in range(cap, w - 1, -1):
            best[c] = max(best[c], best[c - w] + v)
    return best[cap]


@pytest.mark.parametrize("seed", range(6))
def test_two_memory_types_reduce_to_knapsack(seed):
    # fast memory of limited size, slow memory that holds everything: what goes into the fast one is a 0/1
    # knapsack with value = traffic * (1/bw_slow - 1/bw_fast)
    g = RNG(seed)
    T = int(g.integers(4, 10))
    size = g.integers(1, 30, size=T).tolist()
    traffic = (g.random(T) * 100 + 1).tolist()
    cap = int(sum(size) * g.uniform(0.2, 0.7))
    bw = [8.0, 0.05]
    _, t = po.best_assignment(size, traffic, [cap, sum(size)], bw)
    gain = knapsack_max_value(size, [x * (1 / bw[1] - 1 / bw[0]) for x in traffic], cap)
    assert t == pytest.approx(sum(traffic) / bw[1] - gain, rel=1e-12)


def test_hand_worked_case():
    # three tables (size, traffic): A (4, 40), B (3, 36), C (2, 10); fast memory holds 5 at bandwidth 10,
    # slow memory holds everything at bandwidth 1.
    #   fast {A}: 4 + 46 = 50    fast {B}: 3.6 + 50 = 53.6    fast {B, C}: 4.6 + 40 = 44.6    fast {C}: 1 + 76 = 77
    #   {A, B} and {A, C} do not fit.  Best: B and C in the fast memory, 44.6.
    a, t = po.best_assignment([4, 3, 2], [40.0, 36.0, 10.0], [5, 100], [10.0, 1.0])
    assert a == [1, 0, 0] and t == pytest.approx(44.6)


def test_closed_forms():
    size, traffic = [5, 7, 3, 9], [10.0, 3.0, 8.0, 1.0]
    # everything fits the fastest memory
    a, t = po.best_assignment(size, traffic, [100, 100, 100], [4.0, 2.0, 1.0])
    assert a == [0, 0, 0, 0] and t == pytest.approx(sum(traffic) / 4.0)
    # nothing fits anywhere
    a, t = po.best_assignment(size, traffic, [2, 2], [4.0, 1.0])
    assert a is None and math.isinf(t)
    # equal bandwidths: every feasible assignment costs the same
    _, t = po.best_assignment(size, traffic, [12, 12], [2.0, 2.0])
    assert t == pytest.approx(sum(traffic) / 2.0)
    # the time of a given assignment is Eq. 6 term by term
    assert po.lookup_time([0, 1, 1, 0], traffic, [4.0, 0.5]) == pytest.approx(10 / 4 + 3 / 0.5 + 8 / 0.5 + 1 / 4)
    assert not po.feasible([0, 0, 1, 1], size, [11, 100]) and po.feasible([0, 0, 1, 1], size, [12, 12])


