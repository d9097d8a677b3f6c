"""GPU parity of the capacity-bound configuration at the shape bench.py reports.  Its tables take all the pinned
host memory the box allows (64 GiB), so this file is named to be collected before every other GPU test: it then
starts in a process that has pinned nothing yet, and hands the memory back when it is done."""
import pytest

from paper_2305_01515_amd import synth
from parity_util import run_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _hand_pinned_memory_back():
    yield
    import gc
    import torch
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch._C._host_emptyCache()


def test_capacity_bound_at_the_benchmarked_shape():
    """8 tables x dim 128 fp16, 64-way, batch 65536, Poisson(40), Zipf 1.05, 30 % of each batch re-drawn from the
    previous 4 batches (the full per-step shape: 21 M lookups per step); 32 M rows per table instead of 64 M (64 GiB
    of tables: the box refuses to pin more) with a 4 GiB cache (the same 6.25 % of the rows) -- the shape
    `bench.py --workload capacity` reports.  Rows that were looked up are compared against the bar, all others bit
    for bit."""
    cfg = synth.config_capacity(rows=1 << 25, cache_bytes=4 << 30)
    assert cfg.tables[0].cache_slots * 16 == cfg.tables[0].rows and cfg.batch == 65536
    st = run_parity(cfg, steps=3, order="early", oracle_threads=16, init_device="cuda", touched_only=True)
    assert st["total"]["evictions"] > 0 and st["total"]["hits"] > 0
