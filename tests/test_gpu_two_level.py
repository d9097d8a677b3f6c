"""GPU parity of the two-level exclusive cache (Section 5.3, 5.5.4): the HIP library against
the CPU oracle through the C ABI -- both levels' tags and timestamps, all counters and event
sets bit-exact after every batch, pooled outputs and (after flush) all rows and accumulators
within the floating-point bars, for every call order (the race detector of the pipeline)."""
import numpy as np
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import run_parity
from test_gpu_parity import small_cfg

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("factor", [1, 3])
@pytest.mark.parametrize("ways", [1, 8, 64])
def test_small_mixed_model_two_level_serial(ways, factor):
    st = run_parity(small_cfg(synth.FP16, ways, seed=40 + ways), steps=8, order="serial", second_level_factor=factor)
    l2 = st["second_level_total"]
    assert st["total"]["evictions"] > 0 and l2["demotions"] > 0 and l2["hits"] > 0
    if ways == 1:
        assert l2["bypasses"] > 0  # a set of one way is locked by the row that entered it the batch before
    if factor == 1 and ways == 8:
        assert l2["evictions"] > 0


@pytest.mark.parametrize("order", ["inline", "ahead", "early"])
@pytest.mark.parametrize("overlap", [True, False])
def test_two_level_call_orders(order, overlap):
    run_parity(small_cfg(synth.FP32, 16, seed=81), steps=9, order=order, overlap=overlap, second_level_factor=2)


def test_two_level_with_lfu_and_mean():
    run_parity(small_cfg(synth.FP16, 8, seed=82), steps=8, order="ahead", policy="lfu", pooling="mean", second_level_factor=2)


def test_tiny_config_two_level():
    cfg = synth.config_tiny()
    run_parity(cfg, steps=cfg.steps, order="ahead", second_level_factor=2)


def test_main_shape_scaled_two_level():
    # the benchmark workload's shape at 1/16 of the rows and batch; second level four times the first
    cfg = synth.config_main(tables=4, rows=62500, batch=512)
    st = run_parity(cfg, steps=10, order="ahead", second_level_factor=4, check_every=3)
    l2 = st["second_level_total"]
    assert st["total"]["evictions"] > 0 and l2["demotions"] > 0 and l2["hits"] > 0 and st["late_fetches"] > 0


def test_second_level_errors():
    from paper_2305_01515_amd.tbe import TBE, lib
    w = [torch.zeros(100, 8, dtype=torch.float32).pin_memory()]
    m = [torch.zeros(100, dtype=torch.float32).pin_memory()]
    g = TBE(w, m, [16], 4, 8, 64)
    assert lib().tbe_enable_second_level(g._h, 0) == -1
    assert lib().tbe_enable_second_level(g._h, 2) == 0
    assert lib().tbe_enable_second_level(g._h, 2) == -3
    assert lib().tbe_num_sets2(g._h, 0) == 8
    g.close()
    g = TBE(w, m, [0], 4, 8, 64)
    assert lib().tbe_enable_second_level(g._h, 2) == -1  # no first-level cache at all
    idx = torch.tensor([1, 2, 3], device="cuda")
    off = torch.tensor([0, 1, 2, 3, 3, 3, 3, 3, 3], device="cuda")
    g.prefetch(idx, off)
    assert lib().tbe_enable_second_level(g._h, 2) == -3
    g.forward(idx, off)
    g.backward_update(torch.zeros(8, 8, device="cuda"), 0.1, 1e-8)
    g.close()


@pytest.mark.parametrize("factor", [0, 2])
def test_long_run_scaled(factor):
    """40 steps of the benchmark workload's shape at 1/16 of the rows and batch, prefetch ahead and
    pipelined: late rows, skipped write-backs, bypasses and (factor 2) second-level traffic in steady
    state, compared with the oracle every fifth step and after the flush."""
    cfg = synth.config_main(tables=6, rows=62500, batch=512)
    st = run_parity(cfg, steps=40, order="ahead", second_level_factor=factor, check_every=5, oracle_threads=6)
    assert st["late_fetches"] > 0 and st["total"]["bypasses"] > 0 and st["total"]["evictions"] > 0
    if factor:
        l2 = st["second_level_total"]
        assert l2["hits"] > 0 and l2["evictions"] > 0


def test_main_config_full_size_two_level():
    """The benchmark's workload at full size with a second level twice the first, prefetch ahead as
    bench.py issues it, deferred initialisation from NaN-filled tables on top: every prefetch compared."""
    cfg = synth.config_main()
    st = run_parity(cfg, steps=5, order="ahead", oracle_threads=16, init_device="cuda", second_level_factor=2,
                    deferred_init=(7, cfg.init_std))
    l2 = st["second_level_total"]
    assert l2["demotions"] > 0 and l2["hits"] > 0 and st["total"]["bypasses"] > 0 and st["late_fetches"] > 0


@pytest.mark.parametrize("factor", [0, 2])
def test_emulated_slow_backing_tier_changes_nothing_but_time(factor):
    """tbe_set_backing_throttle pauses the host-link kernel after every row it moves to or from the backing
    tier proper (timing only): cache state, events and values stay those of the oracle, with and without a
    second level, prefetch ahead and pipelined; values outside 0 .. 1e8 ns are refused."""
    from paper_2305_01515_amd.tbe import TbeError
    from test_gpu_parity import small_cfg
    st = run_parity(small_cfg(synth.FP16, 8, seed=131), steps=8, order="ahead", second_level_factor=factor,
                    backing_throttle_ns=20000)
    assert st["total"]["evictions"] > 0
    cfg = small_cfg(synth.FP32, 4, seed=132, batch=16)
    from test_gpu_api import make
    g, _, _ = make(cfg, max_lookups=1 << 16)
    for bad in (-1, 10 ** 8 + 1):
        with pytest.raises(TbeError) as e:
            g.set_backing_throttle(bad)
        assert e.value.code == -1
    g.set_backing_throttle(0)
    g.close()
