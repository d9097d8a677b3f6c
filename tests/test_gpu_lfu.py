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
