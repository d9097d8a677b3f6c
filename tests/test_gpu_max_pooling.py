"""GPU parity of max pooling (Section 2.1.1): the HIP library against the CPU oracle through the
C ABI.  Which lookup supplies a maximum is decided on stored values widened exactly, the same
on both sides, and compared element by element (tbe_export_argmax); pooled outputs, updated rows and
accumulators within the floating-point bars.  These fixed cases must compare in full: no step where
the two sides took different rows of a near-tie (parity_util reports that as 'parted_at')."""
import pytest
import torch

from paper_2305_01515_amd import synth
from paper_2305_01515_amd.tbe import TBE, TbeError
from parity_util import run_parity
from test_gpu_parity import small_cfg

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [synth.FP32, synth.FP16])
@pytest.mark.parametrize("ways", [1, 8, 64])
def test_small_mixed_model_max(dtype, ways):
    # fp16 storage makes ties between rows likely (few distinct values): the first lookup of the bag must win
    st = run_parity(small_cfg(dtype, ways, seed=60 + ways), steps=6, order="serial", pooling="max")
    assert st["parted_at"] is None


@pytest.mark.parametrize("order", ["inline", "ahead", "early"])
def test_max_call_orders(order):
    st = run_parity(small_cfg(synth.FP16, 16, seed=84), steps=6, order=order, pooling="max", policy="lfu", second_level_factor=2)
    assert st["parted_at"] is None


def test_max_ragged_batch():
    st = run_parity(small_cfg(synth.FP32, 32, seed=7, batch=1531), steps=3, order="serial", pooling="max")
    assert st["parted_at"] is None


def test_max_with_unpacked_sort_payload():
    # one narrow table and room for 2^27 bags: only 5 bits are left for the position inside a bag, the bags
    # have about 60 lookups, so the batch falls back to plain positions and positions inside the bag are
    # computed from the offsets
    tab = synth.TableCfg(5000, 8, synth.FP16, 1.1, "poisson", 60, 0, 150, cache_slots=7 * 8)
    cfg = synth.WorkloadCfg("narrow", [tab], batch=64, ways=8, steps=3, seed=93, init_std=0.05, lr=0.05)
    st = run_parity(cfg, steps=3, order="ahead", pooling="max", max_batch=1 << 27)
    assert st["parted_at"] is None


def test_main_shape_scaled_max():
    cfg = synth.config_main(tables=4, rows=62500, batch=512)
    st = run_parity(cfg, steps=5, order="ahead", pooling="max", check_every=2)
    assert st["parted_at"] is None


def test_argmax_export_order_errors():
    w = torch.zeros(16, 8, dtype=torch.float16).pin_memory()
    m = torch.zeros(16, dtype=torch.float32).pin_memory()
    idx = torch.tensor([3, 3, 5], device="cuda")
    off = torch.tensor([0, 2, 2, 3], device="cuda")
    g = TBE([w], [m], [8], 4, 3, 8, pooling="max")
    with pytest.raises(TbeError, match="TBE_EORDER"):
        g.argmax(torch.empty(3, 8, dtype=torch.int32, device="cuda"))  # nothing forwarded yet
    g.forward(idx, off)
    a = g.argmax().cpu()
    assert a[0].tolist() == [0] * 8 and a[1].tolist() == [-1] * 8 and a[2].tolist() == [0] * 8
    g.backward_update(torch.zeros(3, 8, device="cuda"), 0.1, 1e-8)
    with pytest.raises(TbeError, match="TBE_EORDER"):
        g.argmax()  # the batch has been updated
    g.close()
    g = TBE([w], [m], [8], 4, 3, 8)
    g.forward(idx, off)
    with pytest.raises(TbeError, match="TBE_EORDER"):
        g.argmax()  # sum pooling keeps no such record
    g.backward_update(torch.zeros(3, 8, device="cuda"), 0.1, 1e-8)
    g.close()
