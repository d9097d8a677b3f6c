"""GPU parity of the LFU replacement policy (Section 5.5.2): the HIP library against the CPU
oracle through the C ABI -- tags, timestamps, per-entry lookup counts, counters and event
sets bit-exact, values within the floating-point bars."""
import numpy as np
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import run_parity
from test_gpu_parity import small_cfg

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [synth.FP32, synth.FP16])
@pytest.mark.parametrize("ways", [1, 8, 32, 64])
def test_small_mixed_model_lfu(dtype, ways):
    st = run_parity(small_cfg(dtype, ways, seed=20 + ways), steps=8, order="serial", policy="lfu")
    assert st["total"]["evictions"] > 0


@pytest.mark.parametrize("order", ["inline", "ahead", "early"])
def test_lfu_call_orders(order):
    run_parity(small_cfg(synth.FP16, 16, seed=78), steps=7, order=order, policy="lfu")


def test_tiny_config_lfu_differs_from_lru():
    cfg = synth.config_tiny()
    lfu = run_parity(cfg, steps=cfg.steps, order="ahead", policy="lfu")
    lru = run_parity(cfg, steps=cfg.steps, order="ahead", policy="lru")
    assert lfu["total"]["uniques"] == lru["total"]["uniques"]
    assert lfu["total"]["hits"] != lru["total"]["hits"]  # the policies keep different rows


def test_main_shape_scaled_lfu():
    # the benchmark workload's shape at 1/16 of the rows and batch: 64 ways, fp16, Poisson pooling
    cfg = synth.config_main(tables=4, rows=62500, batch=512)
    run_parity(cfg, steps=6, order="ahead", policy="lfu", check_every=2)


def test_policy_errors():
    from paper_2305_01515_amd.tbe import TBE, TbeError, lib
    w = [torch.zeros(100, 8, dtype=torch.float32).pin_memory()]
    m = [torch.zeros(100, dtype=torch.float32).pin_memory()]
    g = TBE(w, m, [16], 4, 8, 64)
    assert lib().tbe_set_policy(g._h, 5) == -1
    assert lib().tbe_set_policy(g._h, 1) == 0
    assert lib().tbe_set_policy(g._h, 0) == 0
    idx = torch.tensor([1, 2, 3], device="cuda")
    off = torch.tensor([0, 1, 2, 3, 3, 3, 3, 3, 3], device="cuda")
    g.prefetch(idx, off)
    assert lib().tbe_set_policy(g._h, 1) == -3
    g.forward(idx, off)
    g.backward_update(torch.zeros(8, 8, device="cuda"), 0.1, 1e-8)
    g.flush()
    assert g.cache_freq(0).sum() == 3
    g.close()


def test_lfu_count_saturates_like_the_oracle():
    """Counts near INT32_MAX (put there through the import call on both sides): a hit that would carry the
    count past the limit leaves it at INT32_MAX, and the next miss sees a tie on the count.  One set of two
    ways plus a wider table whose counts are set to random values around the limit."""
    from oracle import Oracle
    from paper_2305_01515_amd.tbe import TBE
    big = np.iinfo(np.int32).max
    rows, dims, slots, ways = [10, 500], [4, 8], [2, 64], 2
    Wn = [np.zeros((r, d), dtype=np.float32) for r, d in zip(rows, dims)]
    Mn = [np.zeros(r, dtype=np.float32) for r in rows]
    Wp = [torch.zeros(r, d, dtype=torch.float32).pin_memory() for r, d in zip(rows, dims)]
    Mp = [torch.zeros(r, dtype=torch.float32).pin_memory() for r in rows]
    o = Oracle(Wn, Mn, slots, ways=ways, policy="lfu")
    g = TBE(Wp, Mp, slots, ways, 1, 4096, policy="lfu")
    rng = np.random.default_rng(5)

    def batch(r0, r1):
        idx = np.array(list(r0) + list(r1), dtype=np.int64)
        off = np.array([0, len(r0), len(idx)], dtype=np.int64)
        o.prefetch(idx, off)
        o.forward()
        o.backward_update(np.zeros((1, 12), dtype=np.float32), 0.01, 1e-8)
        ti, to = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
        g.prefetch(ti, to)
        g.forward(ti, to)
        g.backward_update(torch.zeros(1, 12, device="cuda"), 0.01, 1e-8)
        for t in range(2):
            assert np.array_equal(o.cache_freq(t), g.cache_freq(t)), f"counts of table {t} differ"
            for a, b in zip(o.cache_state(t), g.cache_state(t)):
                assert np.array_equal(a, b)

    wide = lambda n: rng.zipf(1.3, size=n) % 500
    batch([0, 0, 0, 1, 1], wide(600))
    f0 = np.array([big - 2, big - 1], dtype=np.int32)
    f1 = np.where(o.cache_freq(1) > 0, big - rng.integers(0, 6, size=64), 0).astype(np.int32)
    for side in (o, g):
        side.set_cache_freq(0, f0)
        side.set_cache_freq(1, f1)
    batch([0, 0, 0, 0, 0, 1], wide(600))
    assert g.cache_freq(0).tolist() == [big, big] and (g.cache_freq(1) == big).sum() > 0
    batch([2], wide(600))
    assert g.cache_state(0)[0].tolist() == [2, 1]
    batch([3, 3], wide(900))
    g.close()
    o.close()
