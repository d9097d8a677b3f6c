"""The paper's own traffic accounting (host arithmetic only): bench.py takes the forward's Eq. 3 bytes from here.

  Eq. 3 (Section 2.1.2): an embedding lookup moves 2 * D * p bytes -- the row is consumed
      once by forward and once by backward.
  Eq. 4 (Section 4.2): requests that reach the lower tier = requests * alpha, where the
      worked example under the equation fixes alpha as the miss ratio, 1 - hit rate.
"""


def eq3_bytes_per_lookup(dim: int, elem_bytes: int) -> int:
    return 2 * dim * elem_bytes


def eq3_bandwidth(qps: float, tables: int, dim: int, elem_bytes: int, pooling: float) -> float:
    """bytes/s the embedding tables must sustain at `qps` samples per second"""
    return qps * tables * pooling * eq3_bytes_per_lookup(dim, elem_bytes)


def lower_tier_requests(requests: float, hit_rate: float) -> float:
    return requests * (1.0 - hit_rate)
