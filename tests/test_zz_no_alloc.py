"""tbe_backward_update_static (the entry point for callers that cannot allocate: its scratch buffer
is a static array inside the library's device image) against tbe_backward_update, through the C ABI.

Two handles train the same model on the same batches; one takes every backward through
tbe_backward_update, the other through tbe_backward_update_static.  Same kernels, same summation
order: pooled outputs, every row, every accumulator and the cache state must come out bit for bit equal.
The steps are two calls in a row on one GPU, the second with a smaller input (fewer bags, fewer
lookups, fewer partial sums: what the first call left in the shared array must not leak into it); the
tables are small and steep, so several rows have more than 1024 lookups per batch and the partial-sum
buffer really is used.
"""
import numpy as np
import pytest
import torch

from paper_2305_01515_amd import synth
from parity_util import first_bags

pytestmark = pytest.mark.gpu


def _model():
    T = synth.TableCfg
    tabs = [T(3000, 128, synth.FP16, 1.3, "fixed", 24, cache_slots=32 * 40),
            T(2000, 64, synth.FP32, 1.2, "poisson", 30, 1, 100, cache_slots=32 * 30),
            T(5000, 128, synth.FP16, 1.4, "fixed", 16, cache_slots=0)]
    return synth.WorkloadCfg("static-scratch", tabs, batch=2048, ways=32, steps=2, seed=77)


def _train(cfg, batches, sizes, static: bool):
    from paper_2305_01515_amd.tbe import TBE
    Wp, Mp = [], []
    for t, tc in enumerate(cfg.tables):
        w = torch.empty(tc.rows, tc.dim, dtype=torch.float32 if tc.dtype == synth.FP32 else torch.float16, pin_memory=True)
        synth.init_table(cfg, t, device="cpu", out=w)
        Wp.append(w)
        Mp.append(torch.zeros(tc.rows, dtype=torch.float32, pin_memory=True))
    mx = max(int(b[0].numel()) for b in batches) + 1
    g = TBE(Wp, Mp, [tc.cache_slots for tc in cfg.tables], cfg.ways, cfg.batch, mx, overlap=True)
    outs, long_rows = [], []
    for s, (idx, off) in enumerate(batches):
        g.prefetch(idx, off)
        outs.append(g.forward(idx, off).clone())
        go = synth.grad_out(cfg, s + 1)[:sizes[s]].cuda()
        if static:
            g.backward_update_static(go, cfg.lr, cfg.eps)
        else:
            g.backward_update(go, cfg.lr, cfg.eps)
        long_rows.append(g.stats()["last_long_rows"])
    state = [g.cache_state(t) for t in range(cfg.num_tables)]
    g.flush()
    g.close()
    return outs, Wp, Mp, state, long_rows


def test_static_scratch_backward_equals_the_allocating_one_twice_in_a_row():
    cfg = _model()
    stream = synth.BatchStream(cfg, device="cpu")
    full = [stream.next() for _ in range(2)]
    sizes = [cfg.batch, cfg.batch // 3]  # the second call has a smaller input
    batches = [tuple(x.cuda() for x in first_bags(i, f, cfg.num_tables, n)) for (i, f), n in zip(full, sizes)]
    assert batches[1][0].numel() < batches[0][0].numel()
    ref = _train(cfg, batches, sizes, static=False)
    got = _train(cfg, batches, sizes, static=True)
    assert all(n > 0 for n in ref[4]), "the batches have no rows with enough lookups to use the partial sums"
    for s, (a, b) in enumerate(zip(ref[0], got[0])):
        assert torch.equal(a, b), f"pooled output of step {s + 1} differs"
    for t in range(cfg.num_tables):
        assert torch.equal(ref[1][t], got[1][t]), f"rows of table {t} differ"
        assert torch.equal(ref[2][t], got[2][t]), f"accumulators of table {t} differ"
        assert np.array_equal(ref[3][t][0], got[3][t][0]) and np.array_equal(ref[3][t][1], got[3][t][1])


def test_static_scratch_rejects_a_handle_whose_worst_case_does_not_fit():
    from paper_2305_01515_amd.tbe import TBE, TbeError
    w = torch.zeros(1000, 128, dtype=torch.float16, pin_memory=True)
    m = torch.zeros(1000, dtype=torch.float32, pin_memory=True)
    g = TBE([w], [m], [64], 32, 64, 2_000_000, overlap=False)  # 64 x 1954 x 512 B of partial sums: 64 MB
    idx = torch.zeros(64, dtype=torch.int64, device="cuda")
    off = torch.arange(65, dtype=torch.int64, device="cuda")
    g.forward(idx, off)
    go = torch.ones(64, 128, device="cuda")
    with pytest.raises(TbeError) as e:
        g.backward_update_static(go, 0.01, 1e-8)
    assert e.value.code == -5 and "static scratch" in str(e.value)
    g.backward_update(go, 0.01, 1e-8)  # the batch is still there for the allocating call
    g.flush()
    g.close()
    assert float(m[0]) > 0.0
