"""The traffic accounting against the numbers the paper prints (tests/golden/)."""
import os

import pytest

from paper_2305_01515_amd import accounting

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def rows(name):
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].strip()
        if line:
            yield [float(x) for x in line.split()]


def test_eq4_worked_example():
    n = 0
    for req, hit, expect in rows("eq4_lower_tier_requests.txt"):
        assert accounting.lower_tier_requests(req, hit) == pytest.approx(expect, rel=1e-12)
        n += 1
    assert n == 2


def test_eq3_bytes_per_lookup():
    for dim, p, expect in rows("eq3_bandwidth.txt"):
        assert accounting.eq3_bytes_per_lookup(int(dim), int(p)) == expect
    # lookups/s implied by Table 2's bandwidth: BW / (2 D p), e.g. 1300 GB/s at D = 128 fp32
    assert 1300e9 / accounting.eq3_bytes_per_lookup(128, 4) == pytest.approx(1.27e9, rel=0.01)
    assert accounting.eq3_bandwidth(1.0, 1, 128, 4, 33) == 33 * 1024
