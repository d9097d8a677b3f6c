"""GPU tests of the C ABI's contract: error reporting, call order, limits, degenerate
batches, flush as a consistency point, and that overlapping the prefetch with training
changes nothing."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import make_backing, run_parity

pytestmark = pytest.mark.gpu


def little(seed=1, slots=(64, 0), ways=8, dtype=synth.FP32):
    T = synth.TableCfg
    tabs = [T(500, 16, dtype, 1.1, "fixed", 4, cache_slots=slots[0]),
            T(300, 32, dtype, None, "fixed", 2, cache_slots=slots[1])]
    return synth.WorkloadCfg("little", tabs, batch=16, ways=ways, steps=4, seed=seed, init_std=0.1, lr=0.05)


def make(cfg, overlap=True, max_lookups=4096):
    from paper_2305_01515_amd.tbe import TBE
    _, _, Wp, Mp = make_backing(cfg)
    return TBE(Wp, Mp, [t.cache_slots for t in cfg.tables], cfg.ways, cfg.batch, max_lookups, overlap=overlap), Wp, Mp


def batch_of(cfg, step_seed=0):
    s = synth.BatchStream(cfg)
    for _ in range(step_seed + 1):
        idx, off = s.next()
    return idx.cuda(), off.cuda()


def test_out_of_range_index_is_reported_and_harmless():
    from paper_2305_01515_amd.tbe import TbeError
    cfg = little()
    g, Wp, Mp = make(cfg)
    w0 = [w.clone() for w in Wp]
    idx, off = batch_of(cfg)
    bad = idx.clone()
    bad[3] = 500  # table 0 has rows 0..499
    g.prefetch(bad, off)
    out = g.forward(bad, off)
    g.backward_update(torch.ones_like(out), 0.1, 1e-8)
    with pytest.raises(TbeError) as e:
        g.flush()
    assert e.value.code == -2
    with pytest.raises(TbeError):
        g.prefetch(idx, off)  # the error sticks
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(w0, Wp))  # nothing was written
    g.close()


@pytest.mark.parametrize("kind", ["decreasing", "first", "last", "negative"])
def test_bad_offsets_are_reported(kind):
    from paper_2305_01515_amd.tbe import TbeError
    cfg = little()
    g, _, _ = make(cfg)
    idx, off = batch_of(cfg)
    off = off.clone()
    if kind == "decreasing":
        off[5] = off[6] + 1
    elif kind == "first":
        off[0] = 1
    elif kind == "last":
        off[-1] = off[-1] - 1
    else:
        off[2] = -1
    g.prefetch(idx, off)
    with pytest.raises(TbeError) as e:
        g.stats()
    assert e.value.code == -1
    g.close()


def test_call_order_and_limits():
    from paper_2305_01515_amd.tbe import TbeError, lib
    cfg = little()
    g, _, _ = make(cfg, max_lookups=200)
    a, b, c = (batch_of(cfg, i) for i in range(3))
    go = torch.zeros(cfg.batch, cfg.sum_dim, device="cuda")

    def code(fn, *args):
        with pytest.raises(TbeError) as e:
            fn(*args)
        return e.value.code

    assert code(g.backward_update, go, 0.1, 1e-8) == -3      # nothing forwarded
    g.prefetch(*a)
    g.prefetch(*b)                                            # one batch ahead: allowed
    assert code(g.prefetch, *c) == -3                         # two ahead: refused
    assert code(g.flush) == -3                                # batches in flight
    assert code(g.forward, *b) == -6                          # the oldest pending batch is `a`
    out = g.forward(*a)
    assert code(g.forward, *b) == -3                          # `a` not updated yet
    g.backward_update(go, 0.1, 1e-8)
    g.forward(*b)
    g.backward_update(go, 0.1, 1e-8)
    g.flush()
    big_idx = torch.zeros(201, dtype=torch.int64, device="cuda")
    big_off = torch.zeros(2 * cfg.batch + 1, dtype=torch.int64, device="cuda")
    big_off[1:] = 201
    assert code(g.prefetch, big_idx, big_off) == -5           # more lookups than create sized
    wide_off = torch.zeros(2 * (cfg.batch + 1) + 1, dtype=torch.int64, device="cuda")
    assert code(g.prefetch, a[0][:0], wide_off) == -5         # larger batch than create sized
    g.close()
    # tbe_create argument checks
    h = C.c_void_p()
    from paper_2305_01515_amd.tbe import TableSpec
    w = torch.zeros(8, 12, dtype=torch.float16, pin_memory=True)
    m = torch.zeros(8, dtype=torch.float32, pin_memory=True)
    spec = (TableSpec * 1)(TableSpec(8, 12, 1, w.data_ptr(), m.data_ptr(), 0))  # dim 12 is not a multiple of 8
    assert lib().tbe_create(C.byref(h), spec, 1, 8, 4, 16, None, None) == -1
    spec = (TableSpec * 1)(TableSpec(8, 16, 1, w.data_ptr(), m.data_ptr(), 0))
    assert lib().tbe_create(C.byref(h), spec, 1, 65, 4, 16, None, None) == -1
    assert lib().tbe_create(C.byref(h), spec, 1, 0, 4, 16, None, None) == -1


def test_empty_batches():
    cfg = little()
    g, _, _ = make(cfg)
    nb = 2 * cfg.batch
    off = torch.zeros(nb + 1, dtype=torch.int64, device="cuda")
    idx = torch.zeros(0, dtype=torch.int64, device="cuda")
    out = g.forward(idx, off)                                  # no lookups at all
    assert not out.any()
    g.backward_update(torch.ones_like(out), 0.1, 1e-8)
    st = g.stats()["last"]
    assert st["lookups"] == 0 and st["uniques"] == 0
    # every bag empty except the very last one
    idx = torch.tensor([7, 7, 9], dtype=torch.int64, device="cuda")
    off = torch.zeros(nb + 1, dtype=torch.int64, device="cuda")
    off[-1] = 3
    out = g.forward(idx, off)
    torch.cuda.synchronize()
    assert not out[:-1].any() and out[-1, 16:].any() and not out[-1, :16].any()
    g.backward_update(torch.ones_like(out), 0.1, 1e-8)
    g.flush()
    g.close()


@pytest.mark.parametrize("slots", [(0, 0), (504, 304)])
def test_zero_and_full_capacity_against_oracle(slots):
    cfg = little(slots=slots)
    st = run_parity(cfg, steps=5, order="ahead")
    tot = st["total"]
    if slots == (0, 0):
        assert tot["hits"] == 0 and tot["inserts"] == 0 and tot["bypasses"] == tot["uniques"]
    else:
        assert tot["bypasses"] == 0 and tot["evictions"] == 0 and tot["hits"] > 0


def train(cfg, steps, order, overlap, restart_at=None, inputs_ready=False):
    """outputs of every step, final tables, final cache state"""
    from paper_2305_01515_amd.tbe import TBE
    _, _, Wp, Mp = make_backing(cfg)
    slots = [t.cache_slots for t in cfg.tables]
    stream = synth.BatchStream(cfg)
    batches = [tuple(x.cuda() for x in stream.next()) for _ in range(steps)]
    mx = max(int(b[0].numel()) for b in batches) + 1
    g = TBE(Wp, Mp, slots, cfg.ways, cfg.batch, mx, overlap=overlap)
    torch.cuda.synchronize()
    g.set_inputs_ready(inputs_ready)
    outs = []
    for s in range(steps):
        if restart_at is not None and s == restart_at:
            g.flush()
            g.close()
            g = TBE(Wp, Mp, slots, cfg.ways, cfg.batch, mx, overlap=overlap)
        go = synth.grad_out(cfg, s + 1).cuda()
        if order == "serial" or (restart_at is not None and s in (restart_at, restart_at - 1)):
            out = g.forward(*batches[s])
        else:
            if s == 0 or (restart_at is not None and s == restart_at + 1):
                g.prefetch(*batches[s])
            if s + 1 < steps and not (restart_at is not None and s + 1 == restart_at):
                g.prefetch(*batches[s + 1])
            out = g.forward(*batches[s])
        g.backward_update(go, cfg.lr, cfg.eps)
        outs.append(out.cpu())
    state = [g.cache_state(t) for t in range(cfg.num_tables)]
    g.flush()
    g.close()
    return outs, [w.clone() for w in Wp], [m.clone() for m in Mp], state


def mixed(seed):
    T = synth.TableCfg
    tabs = [T(30000, 64, synth.FP16, 1.1, "poisson", 20, 0, 100, cache_slots=16 * 40),
            T(5000, 128, synth.FP32, 1.2, "poisson", 8, 0, 50, cache_slots=16 * 7),
            T(900, 32, synth.FP16, None, "fixed", 3, cache_slots=0)]
    return synth.WorkloadCfg("mixed", tabs, batch=300, ways=16, steps=8, seed=seed, init_std=0.05, lr=0.05)


def test_overlapped_prefetch_is_bitwise_identical_to_serial():
    """The race detector of the stream design: same kernels, same summation order, so
    every output, every row and the cache state must be equal bit for bit."""
    cfg = mixed(5)
    ref = train(cfg, 8, "serial", overlap=False)
    for order, overlap, ready in (("early", True, False), ("early", False, False), ("serial", True, False),
                                  ("early", True, True)):
        got = train(cfg, 8, order, overlap, inputs_ready=ready)
        for a, b in zip(ref[0], got[0]):
            assert torch.equal(a, b)
        for a, b in zip(ref[1] + ref[2], got[1] + got[2]):
            assert torch.equal(a, b)
        for (ta, sa), (tb, sb) in zip(ref[3], got[3]):
            assert np.array_equal(ta, tb) and np.array_equal(sa, sb)


def test_flush_destroy_create_continue():
    """flush is a consistency point: a new handle on the same backing tier continues the
    run with identical outputs and final tables (its cache starts cold)."""
    cfg = mixed(6)
    ref = train(cfg, 8, "early", overlap=True)
    got = train(cfg, 8, "early", overlap=True, restart_at=4)
    for a, b in zip(ref[0], got[0]):
        assert torch.equal(a, b)
    for a, b in zip(ref[1] + ref[2], got[1] + got[2]):
        assert torch.equal(a, b)


def test_repeated_runs_are_reproducible():
    cfg = mixed(7)
    a = train(cfg, 5, "early", overlap=True)
    b = train(cfg, 5, "early", overlap=True)
    assert all(torch.equal(x, y) for x, y in zip(a[0] + a[1] + a[2], b[0] + b[1] + b[2]))


@pytest.mark.parametrize("depth", [2, 5])
def test_prefetch_queue_takes_batches_ahead(depth):
    """With a queue of length `depth` tbe_prefetch accepts that many batches ahead of training; results are
    those of prefetching one batch ahead (the oracle's), the queue refuses one batch too many, flush refuses
    while batches are queued."""
    from paper_2305_01515_amd.tbe import TbeError
    from parity_util import run_parity
    from test_gpu_parity import small_cfg
    run_parity(small_cfg(synth.FP16, 8, seed=95), steps=9, order=f"deep{depth}", second_level_factor=2 if depth == 5 else 0)
    cfg = small_cfg(synth.FP32, 4, seed=96, batch=16)
    g, _, _ = make(cfg, max_lookups=1 << 16)
    stream = synth.BatchStream(cfg, device="cuda")
    bs = [stream.next() for _ in range(depth + 2)]
    g.set_prefetch_queue(depth)
    for b in bs[:depth + 1]:  # the batch about to train and `depth` batches after it
        g.prefetch(*b)
    with pytest.raises(TbeError) as e:
        g.prefetch(*bs[depth + 1])
    assert e.value.code == -3
    with pytest.raises(TbeError):
        g.flush()
    with pytest.raises(TbeError):
        g.set_prefetch_queue(1)
    for b in bs[:depth + 1]:
        g.forward(*b)
        g.backward_update(torch.zeros(cfg.batch, cfg.sum_dim, device="cuda"), 0.1, 1e-8)
    g.flush()
    g.close()


def test_failed_allocation_does_not_leak_into_later_calls():
    """max pooling keeps 4 bytes per pooled element of max_batch bags, three times: for 2^29 bags of 48
    elements that is 309 GB, more than the GPU has.  The refusal
    must name the allocation, and the error must not surface again at the next kernel launch of another handle."""
    from paper_2305_01515_amd.tbe import TBE, TbeError
    cfg = little()
    _, _, Wp, Mp = make_backing(cfg)
    with pytest.raises(TbeError, match="TBE_ENOMEM"):
        TBE(Wp, Mp, [64, 0], cfg.ways, 1 << 29, 4096, pooling="max")
    g = TBE(Wp, Mp, [64, 0], cfg.ways, cfg.batch, 4096)
    idx, off = batch_of(cfg)
    g.prefetch(idx, off)
    g.forward(idx, off)
    g.backward_update(torch.zeros(cfg.batch, 48, device="cuda"), 0.1, 1e-8)
    g.flush()
    g.close()


def test_two_handles_interleaved_equal_each_alone():
    """A model may keep several groups of tables, each behind its own handle, on one GPU.  The handles share
    nothing: driven in turns (and with their prefetches overlapping each other's training) each must produce,
    bit for bit, what it produces alone."""
    from paper_2305_01515_amd.tbe import TBE
    cfgs = [mixed(11), little(seed=12, slots=(64, 32))]
    steps = 6
    alone = [train(c, steps, "early", overlap=True) for c in cfgs]
    run = []
    for c in cfgs:
        _, _, Wp, Mp = make_backing(c)
        stream = synth.BatchStream(c)
        batches = [tuple(x.cuda() for x in stream.next()) for _ in range(steps)]
        mx = max(int(b[0].numel()) for b in batches) + 1
        g = TBE(Wp, Mp, [t.cache_slots for t in c.tables], c.ways, c.batch, mx, overlap=True)
        run.append(dict(cfg=c, Wp=Wp, Mp=Mp, batches=batches, g=g, outs=[]))
    torch.cuda.synchronize()
    for r in run:
        r["g"].prefetch(*r["batches"][0])
    for s in range(steps):
        for r in run:
            if s + 1 < steps:
                r["g"].prefetch(*r["batches"][s + 1])
        for r in run:
            r["outs"].append(r["g"].forward(*r["batches"][s]))
        for r in reversed(run):
            r["g"].backward_update(synth.grad_out(r["cfg"], s + 1).cuda(), r["cfg"].lr, r["cfg"].eps)
    for r, ref in zip(run, alone):
        state = [r["g"].cache_state(t) for t in range(r["cfg"].num_tables)]
        r["g"].flush()
        r["g"].close()
        assert all(torch.equal(a.cpu(), b) for a, b in zip(r["outs"], ref[0]))
        assert all(torch.equal(a, b) for a, b in zip(r["Wp"] + r["Mp"], ref[1] + ref[2]))
        for (ta, sa), (tb, sb) in zip(state, ref[3]):
            assert np.array_equal(ta, tb) and np.array_equal(sa, sb)


def test_binding_keeps_queued_batches_alive_at_depth_four():
    """With four batches accepted ahead of training the library reads a queued batch's index tensors several
    steps after tbe_prefetch returned.  The caller here keeps a batch's tensors only until its forward() call
    and churns the allocator in between (fresh tensors of the same sizes, filled with out-of-range values):
    the binding must hold on to everything the library still reads.  Result: equal, bit for bit, to a run
    whose caller keeps every tensor."""
    cfg = little()
    stream = synth.BatchStream(cfg)
    batches = [stream.next() for _ in range(12)]
    runs = []
    for careless in (False, True):
        g, Wp, Mp = make(cfg)
        g.set_prefetch_queue(4)
        held, pushed, outs, junk = [], 0, [], []
        for s in range(len(batches)):
            while pushed < min(len(batches), s + 5):
                b = tuple(x.cuda().clone() for x in batches[pushed])
                g.prefetch(*b)
                held.append(b)
                pushed += 1
            idx, off = held[0] if careless else held[s]
            out = g.forward(idx, off)
            if careless:
                held.pop(0)
                del idx, off
                junk = [torch.full_like(batches[s][0].cuda(), 1 << 40) for _ in range(4)]
            g.backward_update(synth.grad_out(cfg, s + 1).cuda(), cfg.lr, cfg.eps)
            outs.append(out.clone())
        g.flush()
        g.close()
        runs.append((outs, Wp, Mp))
    a, b = runs
    assert all(torch.equal(x, y) for x, y in zip(a[0], b[0]))
    assert all(torch.equal(x, y) for x, y in zip(a[1] + a[2], b[1] + b[2]))


def test_bad_batch_prefetched_ahead_does_not_lose_the_last_good_batch():
    """A good batch that bypasses rows trains while a batch with an out-of-range index is already prefetched
    behind it.  The bad batch is refused on the device; the good batch's bypassed rows, which were trained on in
    HBM copies, must still reach the backing tier: after the flush (which reports the error) the tables equal
    the oracle's after the good batches."""
    from oracle import Oracle
    from paper_2305_01515_amd.tbe import TbeError
    from parity_util import compare_backing
    cfg = little()
    g, Wp, Mp = make(cfg)
    Wn = [w.numpy().copy() for w in Wp]
    Mn = [m.numpy().copy() for m in Mp]
    o = Oracle(Wn, Mn, [t.cache_slots for t in cfg.tables], cfg.ways)
    stream = synth.BatchStream(cfg)
    good = [stream.next() for _ in range(3)]
    bad_idx, bad_off = stream.next()
    bad_idx = bad_idx.clone()
    bad_idx[0] = cfg.tables[0].rows  # one past the end of table 0
    dev = [tuple(x.cuda() for x in b) for b in good] + [(bad_idx.cuda(), bad_off.cuda())]
    g.prefetch(*dev[0])
    for s in range(3):
        g.prefetch(*dev[s + 1])  # the last one is the bad batch
        g.forward(*dev[s])
        go = synth.grad_out(cfg, s + 1)
        g.backward_update(go.cuda(), cfg.lr, cfg.eps)
        o.prefetch(good[s][0].numpy(), good[s][1].numpy())
        o.forward()
        o.backward_update(go.numpy(), cfg.lr, cfg.eps)
    assert o.stats()[0]["bypasses"] > 0, "the last good batch bypasses no row: the case is not exercised"
    with pytest.raises(TbeError) as e:
        g.flush()
    assert e.value.code == -2
    o.flush()
    compare_backing(cfg, Wn, Mn, Wp, Mp, "after the refused batch")
    g.close()
    o.close()


def test_probe_grouping_takes_1_to_2_pow_30():
    """tbe_set_probe_grouping: a tuning value, refused outside its range"""
    from paper_2305_01515_amd.tbe import TbeError
    from test_gpu_parity import small_cfg
    g, _, _ = make(small_cfg(synth.FP32, 4, seed=5, batch=16), max_lookups=1 << 16)
    for bad in (0, -7, (1 << 30) + 1):
        with pytest.raises(TbeError) as e:
            g.set_probe_grouping(bad)
        assert e.value.code == -1
    g.set_probe_grouping(1)
    g.set_probe_grouping(1 << 30)
    g.close()
