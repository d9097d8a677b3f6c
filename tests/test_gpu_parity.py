"""GPU parity: the HIP library against the CPU oracle, through the C ABI (ctypes)."""
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import run_parity

pytestmark = pytest.mark.gpu


def small_cfg(dtype, ways, seed, batch=96):
    """Mixed little model: dims from 4/8 up to the largest supported, set counts that are
    not powers of two, one table without cache, one fully cached, empty bags, a table
    whose batch overflows its sets (bypass), long runs (hot rows)."""
    epl = 4 if dtype == synth.FP32 else 8
    T = synth.TableCfg
    tabs = [
        T(5000, epl, dtype, 1.05, "poisson", 6, 0, 40, cache_slots=7 * ways),
        T(3001, 64, dtype, 1.2, "poisson", 20, 1, 100, cache_slots=13 * ways),
        T(777, 128, dtype, None, "fixed", 3, cache_slots=0),
        T(4 * ways, 8 * epl, dtype, 0.9, "poisson", 1, 0, 8, cache_slots=4 * ways),
        T(20000, 64 * epl, dtype, 1.3, "poisson", 30, 0, 200, cache_slots=2 * ways),
        T(100000, 24 * epl, dtype, 1.1, "fixed", 11, cache_slots=ways * 301 + 5),
    ]
    return synth.WorkloadCfg("small", tabs, batch=batch, ways=ways, steps=6, seed=seed, init_std=0.05, lr=0.05)


@pytest.mark.parametrize("dtype", [synth.FP32, synth.FP16])
@pytest.mark.parametrize("ways", [1, 8, 32, 64])
def test_small_mixed_model_serial(dtype, ways):
    run_parity(small_cfg(dtype, ways, seed=10 + ways), steps=6, order="serial")


@pytest.mark.parametrize("order", ["inline", "ahead", "early"])
@pytest.mark.parametrize("overlap", [True, False])
def test_small_mixed_model_call_orders(order, overlap):
    run_parity(small_cfg(synth.FP16, 16, seed=77), steps=7, order=order, overlap=overlap)


@pytest.mark.parametrize("second_level_factor", [0, 3])
@pytest.mark.parametrize("policy", ["lru", "lfu"])
@pytest.mark.parametrize("ways", [1, 8, 32, 64])
def test_small_mixed_model_with_grouped_probe(ways, policy, second_level_factor):
    """the probe taking several touched sets per wavefront (as it does by itself only for batches that touch
    thousands of sets): windows that cross tables, contain the rows of the table without cache, sets with
    more misses than ways next to sets with hits only"""
    run_parity(small_cfg(synth.FP16, ways, seed=21 + ways), steps=6, order="ahead", policy=policy,
               second_level_factor=second_level_factor, probe_min_windows=1)


def test_ragged_sizes_span_tiles():
    # more lookups than one sort tile per block and a ragged tail; batch not a multiple of anything
    cfg = small_cfg(synth.FP32, 32, seed=5, batch=1531)
    run_parity(cfg, steps=3, order="serial")


def test_sixteen_lane_rows_at_every_chunk_boundary():
    """Rows of 16 lanes take the forward's unrolled path: a bag is read in chunks of 16 lookups, each chunk in
    two halves of 8.  Fixed bag lengths on both sides of every boundary, rows that fill all 16 lanes and rows
    that leave three idle, both storage types, cached tables and one without a cache (every row read from its
    overflow copy)."""
    T = synth.TableCfg
    lengths = [1, 4, 5, 7, 8, 9, 12, 13, 15, 16, 17, 24, 25, 31, 32, 33]
    tabs = []
    for i, L in enumerate(lengths):
        dtype = synth.FP16 if i % 2 else synth.FP32
        full = 128 if dtype == synth.FP16 else 64
        dim = full if i % 4 < 2 else full * 13 // 16
        tabs.append(T(4000 + 37 * i, dim, dtype, 1.1, "fixed", L, cache_slots=0 if i % 5 == 4 else 16 * (11 + i)))
    cfg = synth.WorkloadCfg("chunks", tabs, batch=50, ways=16, steps=3, seed=41, init_std=0.05, lr=0.05)
    st = run_parity(cfg, steps=3, order="ahead")
    assert st["total"]["bypasses"] > 0 and st["total"]["hits"] > 0


def test_tiny_config_full():
    cfg = synth.config_tiny()
    st = run_parity(cfg, steps=cfg.steps, order="serial")
    assert st["total"]["lookups"] == 20 * 4 * 512 * 20


def test_tiny_config_prefetch_ahead():
    cfg = synth.config_tiny()
    run_parity(cfg, steps=cfg.steps, order="ahead")


def test_small_model_exercises_every_path():
    """the mixed model must actually produce hits, evictions, bypasses and long runs"""
    st = run_parity(small_cfg(synth.FP16, 8, seed=3), steps=6, order="ahead", check_every=2)
    tot = st["total"]
    assert tot["hits"] > 0 and tot["evictions"] > 0 and tot["bypasses"] > 0 and tot["inserts"] > tot["evictions"]
    assert st["h2d_bytes"] > 0 and st["d2h_bytes"] > 0


@pytest.mark.parametrize("second_level_factor", [0, 2])
@pytest.mark.parametrize("ways", [4, 32, 64])
def test_sparse_sets_in_caches_as_large_as_the_tables(ways, second_level_factor):
    """Caches with a slot for every row: a batch touches tens of thousands of sets with one or two rows each, so the
    windows of sets that a wavefront of the probe takes are as long as they get, cross table boundaries, and meet the
    rows of a table without cache and the sets of a cache of two sets in between.  Six steps: free ways filled,
    hits, evictions and bypasses in the small cache, and with a second level rows pushed down and found again."""
    T = synth.TableCfg
    rows = 400_000  # enough touched sets that the probe groups them at all
    full = (rows // ways + 1) * ways
    tabs = [
        T(rows, 32, synth.FP16, 1.05, "poisson", 10, 0, 60, cache_slots=full),
        T(rows, 64, synth.FP16, None, "fixed", 7, cache_slots=full),
        T(5000, 16, synth.FP16, 1.0, "fixed", 3, cache_slots=0),
        T(rows, 32, synth.FP32, 1.1, "poisson", 12, 1, 80, cache_slots=2 * ways),
        T(rows, 128, synth.FP16, 0.9, "poisson", 10, 0, 60, cache_slots=full),
        T(rows, 8, synth.FP32, 1.2, "fixed", 5, cache_slots=rows // 7 // ways * ways),
    ]
    cfg = synth.WorkloadCfg("sparse_sets", tabs, batch=2048, ways=ways, steps=6, seed=77, init_std=0.05, lr=0.05)
    st = run_parity(cfg, steps=6, order="ahead", second_level_factor=second_level_factor)
    tot = st["total"]
    assert tot["hits"] > 0 and tot["evictions"] > 0 and tot["bypasses"] > 0 and tot["inserts"] > 3 * tot["evictions"]


@pytest.mark.parametrize("dtype,dim", [(synth.FP32, 128), (synth.FP16, 64), (synth.FP16, 256)])
@pytest.mark.parametrize("pooling", ["sum", "mean"])
def test_rows_with_a_large_share_of_all_lookups(dtype, dim, pooling):
    """Zipf 1.4 over a single table: one row takes a third of the batch's quarter of a million lookups and a dozen
    more take thousands each.  Such rows enter the heavy rows' kernel in parts of 2048 lookups, and from 512 partial
    sums on their parts are added up side by side, the last part in finishing the row (arrival counters, which must
    be back at zero for the next batch: six steps); a second, ordinary table runs along."""
    T = synth.TableCfg
    tabs = [
        T(200_000, dim, dtype, 1.4, "fixed", 64, cache_slots=32 * 400),
        T(3001, 64, synth.FP16, 1.2, "poisson", 20, 1, 100, cache_slots=32 * 13),
    ]
    cfg = synth.WorkloadCfg("hot_rows", tabs, batch=4096, ways=32, steps=6, seed=500 + dim, init_std=0.05, lr=0.05)
    st = run_parity(cfg, steps=6, order="ahead", pooling=pooling)
    assert st["total"]["hits"] > 0 and st["total"]["inserts"] > 0


def test_main_config_full_size():
    """The benchmark's workload at full size (32 tables x 1M rows x dim 128 fp16, batch
    8192), prefetch issued ahead as bench.py does; 12 steps, every pooled output compared, the cache
    state after every fourth prefetch and the last, all 32M rows after the flush.  Every vector is held
    against the plain bar (2e-3 of the vector's own largest magnitude); the tally printed below says how
    close the worst one came."""
    cfg = synth.config_main()
    st = run_parity(cfg, steps=12, order="ahead", oracle_threads=16, init_device="cuda", check_every=4)
    print("main configuration, 12 steps:", st["tolerance"])
    assert st["total"]["bypasses"] > 0 and st["total"]["evictions"] > 0
    assert st["tolerance"]["vectors_on_peak_scale"] == 0 and st["tolerance"]["worst_error_over_plain_bar"] <= 1.0


@pytest.mark.parametrize("max_batch", [1 << 20, 1 << 27])
def test_sort_payload_with_and_without_the_bag(max_batch):
    """The sort payload carries (bag, position inside the bag) when both fit 32 bits.  The split is
    fixed by tables x max_batch: with 2^20 bags' worth of room the model's bags (up to 200 lookups)
    fit; with 2^27 only bags of up to 4 lookups would, so the batch falls back to plain positions and
    the gathered bag ids.  Both must give the same results."""
    run_parity(small_cfg(synth.FP16, 8, seed=91), steps=4, order="ahead", max_batch=max_batch)


@pytest.mark.parametrize("big_rows,key_bits", [(17_000_000, 25), (40_000_000, 26), (100_000_000, 27), (9_000_000, 24)])
def test_sort_digit_widths_on_small_ragged_batches(big_rows, key_bits):
    """The sort key has as many bits as the keys of all tables need; 25 to 27 bits are sorted in three passes with
    9-bit digits among them, everything else by digits of up to 8 bits.  One table of narrow rows sets the key width
    (its rows are spread over the whole range by uniform indices, so every digit value occurs), small ragged
    batches: tiles that are not full, workgroups without keys."""
    T = synth.TableCfg
    tabs = [
        T(big_rows, 4, synth.FP32, None, "poisson", 9, 0, 50, cache_slots=64 * 8),
        T(3001, 64, synth.FP16, 1.2, "poisson", 20, 1, 100, cache_slots=13 * 8),
        T(777, 128, synth.FP16, None, "fixed", 3, cache_slots=0),
    ]
    assert (sum(t.rows for t in tabs) - 1).bit_length() <= key_bits
    cfg = synth.WorkloadCfg("wide_keys", tabs, batch=611, ways=8, steps=3, seed=300 + key_bits, init_std=0.05, lr=0.05)
    run_parity(cfg, steps=3, order="ahead", init_device="cuda", touched_only=True)


@pytest.mark.parametrize("second_level_factor", [0, 2, 5])
@pytest.mark.parametrize("pooling", ["sum", "max"])
def test_flush_between_steps_then_train_on(second_level_factor, pooling):
    """flush in the middle of training: the backing tier is compared at every flush and training goes on.
    The caches are small against the batches, so rows evicted by the batch before a flush come back right
    after it -- the case where a leftover 'still on its way' mark would make a later write-back be skipped."""
    cfg = small_cfg(synth.FP16, 4, seed=123)
    st = run_parity(cfg, steps=8, order="serial", flush_every=1, second_level_factor=second_level_factor, pooling=pooling)
    assert st["total"]["evictions"] > 0 and st["parted_at"] is None
    run_parity(small_cfg(synth.FP32, 8, seed=124), steps=7, order="inline", flush_every=2, second_level_factor=second_level_factor,
               pooling=pooling, deferred_init=(5, 0.05))
