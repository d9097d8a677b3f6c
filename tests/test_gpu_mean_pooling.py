"""GPU parity of mean pooling (Section 2.1.1): the HIP library against the CPU oracle through
the C ABI; pooled outputs, updated rows and accumulators within the floating-point bars,
cache state bit-exact (it does not depend on the pooling mode)."""
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import run_parity
from test_gpu_parity import small_cfg

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [synth.FP32, synth.FP16])
@pytest.mark.parametrize("ways", [1, 8, 64])
def test_small_mixed_model_mean(dtype, ways):
    # empty bags, one-lookup bags, bags of 200, rows with thousands of lookups (every backward kernel)
    run_parity(small_cfg(dtype, ways, seed=30 + ways), steps=6, order="serial", pooling="mean")


@pytest.mark.parametrize("order", ["inline", "ahead", "early"])
def test_mean_call_orders(order):
    run_parity(small_cfg(synth.FP16, 16, seed=79), steps=6, order=order, pooling="mean", policy="lfu")


def test_mean_ragged_batch():
    run_parity(small_cfg(synth.FP32, 32, seed=6, batch=1531), steps=3, order="serial", pooling="mean")


def test_main_shape_scaled_mean():
    cfg = synth.config_main(tables=4, rows=62500, batch=512)
    run_parity(cfg, steps=5, order="ahead", pooling="mean", check_every=2)


def test_pooling_errors():
    from paper_2305_01515_amd.tbe import TBE, lib
    w = [torch.zeros(100, 8, dtype=torch.float32).pin_memory()]
    m = [torch.zeros(100, dtype=torch.float32).pin_memory()]
    g = TBE(w, m, [16], 4, 8, 64)
    assert lib().tbe_set_pooling(g._h, 3) == -1
    assert lib().tbe_set_pooling(g._h, 1) == 0
    idx = torch.tensor([1, 2, 3], device="cuda")
    off = torch.tensor([0, 1, 2, 3, 3, 3, 3, 3, 3], device="cuda")
    g.prefetch(idx, off)
    assert lib().tbe_set_pooling(g._h, 0) == -3
    g.forward(idx, off)
    g.backward_update(torch.zeros(8, 8, device="cuda"), 0.1, 1e-8)
    g.flush()
    g.close()
