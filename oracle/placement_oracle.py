"""Oracle of the embedding table assignment (paper Section 5.6.1, Eq. 6).  TEST
INFRASTRUCTURE ONLY: tests/ may import it, the product path may not.

The assignment the paper asks its mixed-integer solver for, written out as what it is:
every table goes to exactly one memory type, the tables of a memory type must fit its
size, and among all such assignments the one with the smallest lookup time

    time = sum over memory types m, tables t assigned to m of (D_t * L_t * p_t) / BW_m

is wanted (one GPU here, so the maximum over GPUs in Eq. 6 is over one term).  This file
enumerates all M^T assignments -- usable for about ten tables -- in plain Python floats
(fp64).  `traffic[t]` is the numerator D*L*p of table t (bytes it moves per step),
`size[t]` its bytes, `capacity[m]` / `bandwidth[m]` the memory types.
"""
from itertools import product
from typing import List, Optional, Sequence, Tuple


def lookup_time(assign: Sequence[int], traffic: Sequence[float], bandwidth: Sequence[float]) -> float:
    """Eq. 6 for one GPU."""
    return sum(traffic[t] / bandwidth[m] for t, m in enumerate(assign))


def feasible(assign: Sequence[int], size: Sequence[int], capacity: Sequence[int]) -> bool:
    used = [0] * len(capacity)
    for t, m in enumerate(assign):
        used[m] += size[t]
    return all(u <= c for u, c in zip(used, capacity))


def best_assignment(size: Sequence[int], traffic: Sequence[float], capacity: Sequence[int],
                    bandwidth: Sequence[float]) -> Tuple[Optional[List[int]], float]:
    """(assignment, time) of the best feasible assignment, (None, inf) if none fits.
    Among assignments of equal time the first in enumeration order is returned; only the
    time is unique."""
    best, best_t = None, float("inf")
    for assign in product(range(len(capacity)), repeat=len(size)):
        if not feasible(assign, size, capacity):
            continue
        t = lookup_time(assign, traffic, bandwidth)
        if t < best_t:
            best, best_t = list(assign), t
    return best, best_t
