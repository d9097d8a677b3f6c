"""GPU parity of the pipeline several batches deep (tbe_set_prefetch_depth, Section 5.7): batches are fetched into the
cache up to D ahead of training, the ways of the D batches before the one being decided on are locked.  The oracle
runs the same lock sequentially; cache state, events, counters (bit-exact) and values (the stated bars) must agree."""
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import run_parity
from test_gpu_parity import small_cfg

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("depth", [2, 3])
@pytest.mark.parametrize("dtype,ways", [(synth.FP16, 8), (synth.FP32, 4)])
@pytest.mark.parametrize("overlap", [True, False])
def test_small_model_at_depth(depth, dtype, ways, overlap):
    st = run_parity(small_cfg(dtype, ways, seed=140 + depth), steps=12, order=f"pipe{depth}", overlap=overlap)
    assert st["total"]["bypasses"] > 0 and st["total"]["evictions"] > 0 and st["total"]["hits"] > 0
    # rows that a batch still in flight had bypassed were wanted again and taken from its copies
    assert st["prefetch_depth"] == depth and st["rows_from_copies"] > 0


@pytest.mark.parametrize("seed", range(6))
def test_modes_at_depth(seed):
    """LFU, mean and max pooling, deferred initialisation, an emulated slow tier: each with the deep pipeline."""
    kw = [dict(policy="lfu"), dict(pooling="mean"), dict(pooling="max"), dict(deferred_init=(5, 0.05)),
          dict(backing_throttle_ns=5000), dict(policy="lfu", pooling="mean", deferred_init=(9, 0.02))][seed]
    run_parity(small_cfg(synth.FP16, 8, seed=150 + seed), steps=10, order=f"pipe{2 + seed % 2}", **kw)


def test_benchmark_shape_scaled_at_depth_2():
    """40 steps of the benchmark workload's shape at 1/16 of the rows and batch, two batches deep: late rows from
    parked victims and from overflow copies of batches still in flight, in steady state."""
    cfg = synth.config_main(tables=6, rows=62500, batch=512)
    st = run_parity(cfg, steps=40, order="pipe2", check_every=5, oracle_threads=6)
    assert st["late_fetches"] > 0 and st["total"]["bypasses"] > 0 and st["total"]["evictions"] > 0
    assert st["rows_from_copies"] > 0


def test_depth_is_refused_where_it_cannot_be():
    from paper_2305_01515_amd.tbe import TbeError
    from test_gpu_api import make
    cfg = small_cfg(synth.FP32, 4, seed=160, batch=16)
    g, _, _ = make(cfg, max_lookups=1 << 16)
    for bad in (0, 8):
        with pytest.raises(TbeError) as e:
            g.set_prefetch_depth(bad)
        assert e.value.code == -1
    g.set_prefetch_depth(2)
    with pytest.raises(TbeError) as e:
        g.set_prefetch_depth(3)  # once
    assert e.value.code == -3
    with pytest.raises(TbeError) as e:
        g.set_prefetch_queue(4)
    assert e.value.code == -3
    stream = synth.BatchStream(cfg, device="cuda")
    bs = [stream.next() for _ in range(5)]
    for b in bs[:3]:  # the batch about to train and two beyond it
        g.prefetch(*b)
    with pytest.raises(TbeError) as e:
        g.prefetch(*bs[3])
    assert e.value.code == -3
    for b in bs[:3]:
        g.forward(*b)
        g.backward_update(torch.zeros(cfg.batch, cfg.sum_dim, device="cuda"), 0.1, 1e-8)
    g.flush()
    g.close()
    g, _, _ = make(cfg, max_lookups=1 << 16)
    g.prefetch(*bs[0])
    with pytest.raises(TbeError) as e:
        g.set_prefetch_depth(2)  # after the first batch
    assert e.value.code == -3
    g.forward(*bs[0])
    g.backward_update(torch.zeros(cfg.batch, cfg.sum_dim, device="cuda"), 0.1, 1e-8)
    g.close()


@pytest.mark.parametrize("seed", range(40))
def test_random_model_at_random_depth(seed):
    """Randomised models (table count, rows, dims, storage types, ways 1..64, cache sizes including none and more
    than the rows, batch, pooling, skew) at depth 2..5 with LFU / LRU, every pooling mode, deferred initialisation,
    batches of varying size and refused calls in between."""
    import numpy as np
    from test_gpu_fuzz import draw
    cfg, _, overlap = draw(300 + seed)
    g = np.random.default_rng(seed)
    kw = dict(policy=str(g.choice(["lru", "lfu"])), pooling=str(g.choice(["sum", "mean", "max"])),
              deferred_init=(seed, 0.05) if g.integers(0, 2) else None)
    if g.integers(0, 3) == 0:
        kw["vary_batch"] = seed + 2
    if g.integers(0, 2):
        kw["misuse"] = seed + 1
    run_parity(cfg, steps=int(g.integers(4, 11)), order="pipe%d" % int(g.integers(2, 6)), overlap=overlap, **kw)


def test_main_config_full_size_at_depth_2():
    """The benchmark workload at full size (32 tables x 1M rows x dim 128 fp16, batch 8192, 64-way cache of 5 %), two
    batches deep as `bench.py --prefetch-depth 2` issues it: every prefetch compared with the oracle's."""
    cfg = synth.config_main()
    st = run_parity(cfg, steps=6, order="pipe2", oracle_threads=16, init_device="cuda")
    assert st["total"]["bypasses"] > 0 and st["late_fetches"] > 0 and st["rows_from_copies"] > 0
    assert st["tolerance"]["vectors_on_peak_scale"] == 0


def test_bad_batch_prefetched_two_ahead_loses_nothing():
    """Two batches deep; the second batch beyond the one in training has an index out of range and is refused on
    the device.  The batches in front of it train on; after the flush (which reports the error) the tables equal
    the locked oracle's after the good batches -- bypassed rows, which train in copies outside the cache, included."""
    from oracle import Oracle
    from paper_2305_01515_amd.tbe import TbeError
    from parity_util import compare_backing
    from test_gpu_api import little, make
    cfg = little()
    g, Wp, Mp = make(cfg)
    g.set_prefetch_depth(2)
    Wn = [w.numpy().copy() for w in Wp]
    Mn = [m.numpy().copy() for m in Mp]
    o = Oracle(Wn, Mn, [t.cache_slots for t in cfg.tables], cfg.ways, prefetch_lock=2)
    stream = synth.BatchStream(cfg)
    good = [stream.next() for _ in range(4)]
    bad_idx, bad_off = stream.next()
    bad_idx = bad_idx.clone()
    bad_idx[0] = cfg.tables[0].rows  # one past the end of table 0
    dev = [tuple(x.cuda() for x in b) for b in good] + [(bad_idx.cuda(), bad_off.cuda())]
    g.prefetch(*dev[0])
    g.prefetch(*dev[1])
    bypasses = 0
    for s in range(4):
        if s + 2 < len(dev):
            g.prefetch(*dev[s + 2])  # the last one is the bad batch
        g.forward(*dev[s])
        go = synth.grad_out(cfg, s + 1)
        g.backward_update(go.cuda(), cfg.lr, cfg.eps)
        o.prefetch(good[s][0].numpy(), good[s][1].numpy())
        o.forward()
        o.backward_update(go.numpy(), cfg.lr, cfg.eps)
        bypasses += o.stats()[0]["bypasses"]
    assert bypasses > 0, "no good batch bypasses a row: the case is not exercised"
    with pytest.raises(TbeError) as e:
        g.flush()
    assert e.value.code == -2
    o.flush()
    compare_backing(cfg, Wn, Mn, Wp, Mp, "after the refused batch")
    g.close()
    o.close()


def test_heterogeneous_model_scaled_at_depth_3():
    """100 tables of three widths (8, 16 and 32 lanes per row), pooling means 1..100, skews 0.9..1.3, rows 1/100 of
    the configuration's and batch 2048, three batches deep: every backward class and table class under the lock."""
    cfg = synth.config_hetero(max_rows=5e5, batch=2048, cache_bytes=160 << 20)
    probe = synth.BatchStream(cfg)
    _, off = probe.next()
    lookups = [int(off[(t + 1) * cfg.batch] - off[t * cfg.batch]) for t in range(cfg.num_tables)]
    synth.split_cache_budget(cfg, lookups, cfg.cache_bytes)
    st = run_parity(cfg, steps=8, order="pipe3", oracle_threads=16, init_device="cuda")
    assert st["total"]["hits"] > 0 and st["total"]["inserts"] > 0 and st["rows_from_copies"] > 0
