"""Randomised parity: small models drawn from a seed (table count, rows, dims, storage
types, ways, cache sizes incl. none and more than the rows, batch, pooling, skew, call
order) against the oracle.  Each case is a few thousand lookups; the shapes hit group sizes
from 1 to 64 lanes, set counts that are not powers of two, and every backward class."""
import numpy as np
import pytest

from paper_2305_01515_amd import synth
from parity_util import run_parity

pytestmark = pytest.mark.gpu


def draw(seed):
    g = np.random.default_rng(seed)
    ways = int(g.choice([1, 2, 3, 7, 16, 32, 33, 64]))
    T = int(g.integers(1, 7))
    tabs = []
    for _ in range(T):
        dtype = int(g.integers(0, 2))
        epl = 4 if dtype == synth.FP32 else 8
        dim = epl * int(g.choice([1, 2, 3, 5, 8, 16, 24, 32, 64]))
        rows = int(g.choice([1, 5, 63, 500, 4097, 30000]))
        kind = g.choice(["none", "tiny", "some", "all"])
        slots = {"none": 0, "tiny": ways, "some": max(ways, rows // 7), "all": rows + 3 * ways}[str(kind)]
        alpha = [None, 0.8, 1.0, 1.3][int(g.integers(0, 4))]
        if g.random() < 0.5:
            pool = ("fixed", int(g.integers(0, 40)))
        else:
            pool = ("poisson", float(g.choice([0.3, 2.0, 15.0, 60.0])))
        tabs.append(synth.TableCfg(rows, dim, dtype, alpha, pool[0], pool[1], 0, 150, cache_slots=int(slots)))
    batch = int(g.choice([1, 2, 17, 64, 300]))
    order = str(g.choice(["serial", "inline", "ahead", "early"]))
    overlap = bool(g.integers(0, 2))
    cfg = synth.WorkloadCfg(f"fuzz{seed}", tabs, batch=batch, ways=ways, steps=4, seed=1000 + seed, init_std=0.05, lr=0.05)
    return cfg, order, overlap


@pytest.mark.parametrize("seed", range(24))
def test_random_model(seed):
    cfg, order, overlap = draw(seed)
    # every other draw with the probe grouping touched sets as it does for large batches
    run_parity(cfg, steps=4, order=order, overlap=overlap, probe_min_windows=seed % 2)


@pytest.mark.parametrize("seed", range(24))
def test_random_model_two_level(seed):
    """the same draws with a second-level cache, LFU or LRU and sum or mean pooling, more steps
    (rows must be pushed down, found again, and pushed out of the second level)"""
    cfg, order, overlap = draw(100 + seed)
    if not any(t.cache_slots >= cfg.ways for t in cfg.tables):
        cfg.tables[0].cache_slots = cfg.ways
    g = np.random.default_rng(seed)
    run_parity(cfg, steps=7, order=order, overlap=overlap, second_level_factor=int(g.choice([1, 2, 5])),
               policy=str(g.choice(["lru", "lfu"])), pooling=str(g.choice(["sum", "mean", "max"])),
               probe_min_windows=(seed + 1) % 2)


def draw_options(seed):
    """every option of the library at once: a model as above plus second level, policy, pooling, deferred
    initialisation, a deeper prefetch queue, flushes between steps, the width of the sort payload, and calls
    that must be refused sprinkled in between, batches of varying size"""
    cfg, order, overlap = draw(seed)
    g = np.random.default_rng(seed)
    two = bool(g.integers(0, 2))
    if two and not any(t.cache_slots >= cfg.ways for t in cfg.tables):
        cfg.tables[0].cache_slots = cfg.ways
    kw = dict(second_level_factor=int(g.choice([1, 2, 5])) if two else 0, policy=str(g.choice(["lru", "lfu"])),
              pooling=str(g.choice(["sum", "mean", "max"])), deferred_init=(seed, 0.05) if g.integers(0, 2) else None)
    if g.integers(0, 4) == 0:
        order = "deep%d" % int(g.integers(2, 5))
    steps = int(g.integers(3, 9))
    if order in ("serial", "inline") and g.integers(0, 2):
        kw["flush_every"] = int(g.integers(1, 4))
    if g.integers(0, 3) == 0:
        kw["max_batch"] = int(g.choice([cfg.batch, 1 << 20, 1 << 27]))
        if kw["pooling"] == "max":  # max pooling keeps 4 bytes per pooled element of max_batch bags, three times
            kw["max_batch"] = min(kw["max_batch"], max(cfg.batch, (1 << 30) // sum(t.dim for t in cfg.tables)))
    if g.integers(0, 2):
        kw["misuse"] = seed + 1  # refused calls in between, see parity_util.run_parity
    if g.integers(0, 3) == 0:
        kw["vary_batch"] = seed + 2  # a different number of bags every step
    return cfg, dict(steps=steps, order=order, overlap=overlap, **kw)


@pytest.mark.parametrize("seed", range(5000, 5032))
def test_random_model_every_option(seed):
    cfg, kw = draw_options(seed)
    run_parity(cfg, **kw)
