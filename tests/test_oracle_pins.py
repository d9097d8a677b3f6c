"""Pins of the CPU oracle against things other than itself: library routines
(torch embedding_bag, autograd, torch.optim.Adagrad, numpy float16), closed
forms, the invariants a cache must satisfy, and independent brute-force LRU
models written here in plain Python.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import Oracle, OracleError, lib

RNG = np.random.default_rng


def make_tables(rows, dims, dtypes, seed=0, std=0.1):
    g = RNG(seed)
    W = [(g.standard_normal((r, d)) * std).astype(dt) for r, d, dt in zip(rows, dims, dtypes)]
    M = [np.zeros(r, dtype=np.float32) for r in rows]
    return W, M


def random_batch(rows, B, L, seed, skew=True):
    """indices/offsets for len(rows) tables, bag lengths in [0, 2L]."""
    g = RNG(seed)
    idx, lens = [], []
    for H in rows:
        ln = g.integers(0, 2 * L + 1, size=B)
        n = int(ln.sum())
        if skew:
            r = np.minimum((g.pareto(1.0, size=n)).astype(np.int64), H - 1)
            r = (r * 7919 + 13) % H
        else:
            r = g.integers(0, H, size=n)
        idx.append(r.astype(np.int64))
        lens.append(ln)
    lens = np.concatenate(lens)
    off = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    return np.concatenate(idx), off


# ----------------------------------------------------------------------------
# fp16 conversion: against numpy's float16
# ----------------------------------------------------------------------------

def test_half_conversion_matches_numpy():
    g = RNG(1)
    xs = np.concatenate([
        g.standard_normal(20000) * 10.0 ** g.integers(-9, 5, size=20000),
        np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 70000.0, -70000.0, 2.0 ** -24, 2.0 ** -25,
                  2.0 ** -25 * 1.0000001, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11,
                  1.0 + 2.0 ** -11 + 2.0 ** -30, 1.0 + 3 * 2.0 ** -11, 6.1e-5, 5.9e-8, 2.9e-8, 3.1e-8]),
    ])
    with np.errstate(over="ignore"):
        ref = xs.astype(np.float16).view(np.uint16)
    got = np.array([lib().orc_double_to_half(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(ref, got)
    allh = np.arange(0, 65536, dtype=np.uint16)
    back = np.array([lib().orc_half_to_double(int(h)) for h in allh])
    refb = allh.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(back), np.isnan(refb))
    ok = ~np.isnan(refb)
    assert np.array_equal(back[ok], refb[ok])


# ----------------------------------------------------------------------------
# forward: torch's embedding_bag in fp64, and a hand-computed case
# ----------------------------------------------------------------------------

def torch_forward(W, idx, off, B):
    outs, T = [], len(W)
    for t in range(T):
        lo, hi = off[t * B], off[(t + 1) * B]
        o = torch.from_numpy(off[t * B:(t + 1) * B] - lo)
        i = torch.from_numpy(idx[lo:hi])
        w = torch.from_numpy(W[t].astype(np.float64))
        outs.append(torch.nn.functional.embedding_bag(i, w, o, mode="sum"))
    return torch.cat(outs, dim=1).numpy()


@pytest.mark.parametrize("slots", [0, 64, 4096])
@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_forward_matches_embedding_bag(slots, dt):
    rows, dims = [1000, 333, 4096], [8, 16, 4]
    W, M = make_tables(rows, dims, [dt] * 3, seed=3)
    W0 = [w.copy() for w in W]
    o = Oracle(W, M, [slots] * 3, ways=8)
    B = 37
    for step in range(3):
        idx, off = random_batch(rows, B, 6, seed=10 + step)
        o.prefetch(idx, off)
        out = o.forward()
        ref = torch_forward(W0, idx, off, B)  # no update was applied: rows keep their initial values
        assert np.array_equal(out, ref.astype(np.float32))


def test_forward_hand_example():
    # one table, 3 rows, dim 2; bags: {0,2,2}, {}, {1}
    W = [np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]], dtype=np.float32)]
    M = [np.zeros(3, dtype=np.float32)]
    o = Oracle(W, M, [2], ways=2)
    o.prefetch(np.array([0, 2, 2, 1]), np.array([0, 3, 3, 4]))
    out = o.forward()
    assert out.tolist() == [[201.0, 402.0], [0.0, 0.0], [10.0, 20.0]]


# ----------------------------------------------------------------------------
# backward + row-wise Adagrad
# ----------------------------------------------------------------------------

def test_dim1_is_elementwise_adagrad():
    """With D = 1 a row-wise accumulator is an element-wise one, so the dense
    torch.optim.Adagrad on a [H, 1] parameter is the reference; the gradient of
    each row comes from autograd through embedding_bag."""
    H, B, lr, eps = 50, 16, 0.05, 1e-3
    W, M = make_tables([H], [1], [np.float32], seed=5, std=1.0)
    p = torch.nn.Parameter(torch.from_numpy(W[0].astype(np.float64)))
    opt = torch.optim.Adagrad([p], lr=lr, lr_decay=0, weight_decay=0, initial_accumulator_value=0, eps=eps)
    o = Oracle(W, M, [16], ways=4)
    for step in range(6):
        idx, off = random_batch([H], B, 4, seed=20 + step)
        go = RNG(30 + step).standard_normal((B, 1)).astype(np.float32)
        o.prefetch(idx, off)
        out = o.forward()
        opt.zero_grad()
        ref_out = torch.nn.functional.embedding_bag(torch.from_numpy(idx), p, torch.from_numpy(off[:-1]), mode="sum")
        # the oracle stores rows as fp32 between steps, torch keeps fp64: allow storage rounding
        np.testing.assert_allclose(out, ref_out.detach().numpy(), rtol=1e-6, atol=2e-6)
        (ref_out * torch.from_numpy(go.astype(np.float64))).sum().backward()
        opt.step()
        o.backward_update(go, lr, eps)
    o.flush()
    np.testing.assert_allclose(W[0], p.detach().numpy(), rtol=2e-6, atol=1e-6)
    np.testing.assert_allclose(M[0], opt.state[p]["sum"].numpy()[:, 0], rtol=2e-6, atol=1e-9)
    assert (M[0] > 0).sum() > 10 and (M[0] == 0).sum() > 0  # touched and untouched rows both occur


def test_first_update_closed_form():
    """From m = 0 a row with gradient g becomes w - lr * g / (|g|_2 / sqrt(D) + eps)."""
    D, lr, eps = 8, 0.1, 1e-2
    W, M = make_tables([10], [D], [np.float32], seed=7, std=1.0)
    W0 = W[0].copy()
    o = Oracle(W, M, [0], ways=4)
    go = RNG(8).standard_normal((2, D)).astype(np.float32)
    # bag 0 = {3, 3, 5}, bag 1 = {3}: row 3 receives 2*go[0] + go[1], row 5 receives go[0]
    o.prefetch(np.array([3, 3, 5, 3]), np.array([0, 3, 4]))
    o.forward()
    o.backward_update(go, lr, eps)
    g3 = 2.0 * go[0].astype(np.float64) + go[1]
    g5 = go[0].astype(np.float64)
    for r, g in ((3, g3), (5, g5)):
        exp = W0[r] - lr * g / (np.linalg.norm(g) / math.sqrt(D) + eps)
        np.testing.assert_allclose(W[0][r], exp, rtol=1e-6)
        np.testing.assert_allclose(M[0][r], (g * g).mean(), rtol=1e-6)
    untouched = [r for r in range(10) if r not in (3, 5)]
    assert np.array_equal(W[0][untouched], W0[untouched]) and not M[0][untouched].any()


def test_gradient_aggregation_matches_autograd():
    """Duplicates inside a bag and across bags: the per-row gradient is what autograd
    gives for sum-pooling; checked through the accumulator m = mean(g^2) and the row."""
    rows, dims, B, lr, eps = [40, 25], [4, 8], 12, 0.01, 1e-8
    W, M = make_tables(rows, dims, [np.float32] * 2, seed=9, std=1.0)
    W0 = [w.copy() for w in W]
    idx, off = random_batch(rows, B, 5, seed=11)
    go = RNG(12).standard_normal((B, sum(dims))).astype(np.float32)
    o = Oracle(W, M, [8, 0], ways=4)
    o.prefetch(idx, off)
    o.forward()
    o.backward_update(go, lr, eps)
    o.flush()
    col = 0
    for t in range(2):
        p = torch.from_numpy(W0[t].astype(np.float64)).requires_grad_()
        lo, hi = off[t * B], off[(t + 1) * B]
        out = torch.nn.functional.embedding_bag(torch.from_numpy(idx[lo:hi]), p,
                                                torch.from_numpy(off[t * B:(t + 1) * B] - lo), mode="sum")
        (out * torch.from_numpy(go[:, col:col + dims[t]].astype(np.float64))).sum().backward()
        g = p.grad.numpy()
        m = (g * g).mean(axis=1)
        np.testing.assert_allclose(M[t], m, rtol=1e-6, atol=1e-12)
        exp = W0[t] - lr * g / (np.sqrt(m)[:, None] + eps)
        np.testing.assert_allclose(W[t], exp, rtol=1e-6, atol=1e-9)
        col += dims[t]


def run_training(slots, ways, dt, steps=8, seed=0, rows=(600, 257, 64), dims=(8, 4, 16), B=24, L=5, flush=True):
    W, M = make_tables(rows, dims, [dt] * len(rows), seed=seed)
    o = Oracle(W, M, slots, ways=ways)
    outs, stats = [], []
    for s in range(steps):
        idx, off = random_batch(rows, B, L, seed=100 + s)
        go = RNG(200 + s).standard_normal((B, sum(dims))).astype(np.float32)
        o.prefetch(idx, off)
        stats.append(o.stats()[0])
        outs.append(o.forward())
        o.backward_update(go, 0.05, 1e-8)
    if flush:
        o.flush()
    return W, M, outs, stats, o


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_results_do_not_depend_on_cache_size(dt):
    """The cache is a performance device: pooled outputs of every step and the final
    tables after flush are bit-identical for no cache, a small one and a full one."""
    rows = (600, 257, 64)
    ref = run_training([0, 0, 0], 4, dt)
    for slots, ways in (([16, 8, 4], 4), ([64, 64, 64], 8), ([640, 264, 64], 8), ([3, 5, 1], 1)):
        got = run_training(slots, ways, dt)
        for a, b in zip(ref[2], got[2]):
            assert np.array_equal(a, b)
        for t in range(len(rows)):
            assert np.array_equal(ref[0][t], got[0][t]) and np.array_equal(ref[1][t], got[1][t])


def test_write_back_not_write_through():
    """Before flush the lower tier is stale for rows that are cached and trained on."""
    W, M, _, _, o = run_training([640, 264, 64], 8, np.float32, flush=False)
    Wf, Mf, _, _, _ = run_training([640, 264, 64], 8, np.float32, flush=True)
    assert any(not np.array_equal(a, b) for a, b in zip(W, Wf))
    # ... but the value "wherever it lives" is current
    for t, r in ((0, 13), (1, 20), (2, 5)):
        w, m = o.read_row(t, r)
        assert np.array_equal(w.astype(np.float32), Wf[t][r]) and m == Mf[t][r]
    o.flush()
    for a, b in zip(W + M, Wf + Mf):
        assert np.array_equal(a, b)


def test_full_capacity_misses_only_on_first_touch():
    rows = (600, 257, 64)
    ways = 8
    slots = [((r + ways - 1) // ways) * ways for r in rows]  # sets*ways >= rows, <= ways rows per set
    _, _, _, stats, o = run_training(slots, ways, np.float32, steps=12)
    seen = [set() for _ in rows]
    W, M = make_tables(rows, (8, 4, 16), [np.float32] * 3)
    o = Oracle(W, M, slots, ways=ways)
    for s in range(12):
        idx, off = random_batch(rows, 24, 5, seed=100 + s)
        o.prefetch(idx, off)
        st = o.stats()[0]
        new = 0
        for t in range(3):
            u = set(idx[off[t * 24]:off[(t + 1) * 24]].tolist())
            new += len(u - seen[t])
            seen[t] |= u
        assert st["inserts"] == new and st["evictions"] == 0 and st["bypasses"] == 0
        assert st["hits"] == st["uniques"] - new


def test_zero_capacity_always_misses():
    _, _, _, stats, o = run_training([0, 0, 0], 4, np.float32)
    for st in stats:
        assert st["hits"] == 0 and st["inserts"] == 0 and st["bypasses"] == st["uniques"] > 0
        assert st["hit_lookups"] == 0
    # fewer slots than one set also means no cache
    _, _, _, stats, _ = run_training([3, 3, 3], 4, np.float32)
    assert all(st["bypasses"] == st["uniques"] for st in stats)


def test_counts_add_up_and_events_match_counts():
    rows = (600, 257, 64)
    W, M = make_tables(rows, (8, 4, 16), [np.float32] * 3)
    o = Oracle(W, M, [32, 16, 8], ways=4)
    for s in range(10):
        idx, off = random_batch(rows, 24, 5, seed=100 + s)
        o.prefetch(idx, off)
        st = o.stats()[0]
        uniq = sum(len(set(idx[off[t * 24]:off[(t + 1) * 24]].tolist())) for t in range(3))
        assert st["uniques"] == uniq and st["lookups"] == idx.size
        assert st["hits"] + st["inserts"] + st["bypasses"] == uniq
        ht, hr = o.events("hit")
        it, ir, isl, iold = o.events("insert")
        bt, br = o.events("bypass")
        assert (len(hr), len(ir), len(br)) == (st["hits"], st["inserts"], st["bypasses"])
        assert int((iold >= 0).sum()) == st["evictions"]
        # lookup-weighted hits: count lookups whose row is in the hit list
        hl = 0
        for t in range(3):
            hs = set(hr[ht == t].tolist())
            hl += sum(1 for r in idx[off[t * 24]:off[(t + 1) * 24]].tolist() if r in hs)
        assert hl == st["hit_lookups"]
        o.forward()
        o.backward_update(np.zeros((24, 28), dtype=np.float32), 0.1, 1e-8)


# ----------------------------------------------------------------------------
# cache state: independent brute-force models
# ----------------------------------------------------------------------------

class ListSetModel:
    """Per set an explicit list of [way, tag, ts]; a batch stamps hits, then gives the
    misses (ascending) the entries in order of (ts, way) among those older than k."""

    def __init__(self, sets, ways):
        self.sets, self.ways = sets, ways
        self.s = [[[w, -1, -1] for w in range(ways)] for _ in range(sets)]

    def batch(self, rows, k):
        hits, ins, byp = [], [], []
        by_set = {}
        for r in sorted(set(rows)):
            by_set.setdefault(r % self.sets if self.sets else -1, []).append(r)
        for s, q in by_set.items():
            if s < 0:
                byp += q
                continue
            ent = self.s[s]
            present = {e[1]: e for e in ent if e[1] >= 0}
            miss = []
            for r in q:
                if r in present:
                    present[r][2] = k
                    hits.append(r)
                else:
                    miss.append(r)
            order = sorted((e for e in ent if e[2] < k), key=lambda e: (e[2], e[0]))
            for j, r in enumerate(miss):
                if j < len(order):
                    e = order[j]
                    ins.append((r, s * self.ways + e[0], e[1]))
                    e[1], e[2] = r, k
                else:
                    byp.append(r)
        return sorted(hits), sorted(ins), sorted(byp)

    def state(self):
        tags = np.array([e[1] for s in self.s for e in sorted(s)], dtype=np.int64)
        ts = np.array([e[2] for s in self.s for e in sorted(s)], dtype=np.int32)
        return tags, ts


@pytest.mark.parametrize("sets,ways,H,n", [(1, 4, 40, 6), (3, 2, 50, 9), (5, 8, 200, 60), (7, 3, 64, 40), (2, 64, 4000, 150)])
def test_cache_state_matches_list_model(sets, ways, H, n):
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [sets * ways], ways=ways)
    model = ListSetModel(sets, ways)
    g = RNG(sets * 100 + ways)
    for k in range(1, 40):
        m = int(g.integers(1, n + 1))
        rows = np.minimum(g.pareto(0.7, size=m).astype(np.int64) * 3 + g.integers(0, 3, size=m), H - 1)
        o.prefetch(rows, np.array([0, m]))
        hits, ins, byp = model.batch(rows.tolist(), k)
        _, hr = o.events("hit")
        _, ir, isl, iold = o.events("insert")
        _, br = o.events("bypass")
        assert sorted(hr.tolist()) == hits
        assert sorted(zip(ir.tolist(), isl.tolist(), iold.tolist())) == ins
        assert sorted(br.tolist()) == byp
        tags, ts = o.cache_state(0)
        mt, mts = model.state()
        assert np.array_equal(tags, mt) and np.array_equal(ts, mts)
        # pipelining invariant (Section 5.7): every row of batch k is resident with ts = k or bypassed
        resident = set(tags[ts == k].tolist())
        assert resident == set(rows.tolist()) - set(byp)


def test_single_lookup_batches_are_textbook_lru():
    """One lookup per batch: no ties among used entries, so each set behaves like a
    move-to-front list of at most W rows."""
    sets, ways, H = 3, 4, 60
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [sets * ways], ways=ways)
    mtf = [[] for _ in range(sets)]
    g = RNG(42)
    for k in range(1, 400):
        r = int(g.integers(0, H) if k % 3 else g.integers(0, 12))
        o.prefetch(np.array([r]), np.array([0, 1]))
        lst = mtf[r % sets]
        st = o.stats()[0]
        if r in lst:
            lst.remove(r)
            assert st["hits"] == 1
        else:
            assert st["inserts"] == 1 and st["bypasses"] == 0
            _, _, _, old = o.events("insert")
            if len(lst) == ways:
                assert old[0] == lst.pop()  # the least recently used row leaves
            else:
                assert old[0] == -1
        lst.insert(0, r)
        tags, _ = o.cache_state(0)
        for s in range(sets):
            assert set(tags[s * ways:(s + 1) * ways].tolist()) - {-1} == set(mtf[s])


def test_overflowing_set_bypasses_highest_rows():
    # one set of 2 ways, batch with 4 distinct rows: the two smallest are inserted
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [2], ways=2)
    o.prefetch(np.array([7, 1, 5, 3, 1]), np.array([0, 5]))
    _, ir, isl, _ = o.events("insert")
    _, br = o.events("bypass")
    assert ir.tolist() == [1, 3] and isl.tolist() == [0, 1] and br.tolist() == [5, 7]
    # next batch: 5 hits nothing; 1 is a hit and keeps its way; 5 replaces row 3 (older stamp)
    o.forward(); o.backward_update(np.zeros((1, 4), dtype=np.float32), 0.1, 1e-8)
    o.prefetch(np.array([5, 1]), np.array([0, 2]))
    tags, ts = o.cache_state(0)
    assert tags.tolist() == [1, 5] and ts.tolist() == [2, 2]


def test_errors():
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [4], ways=2)
    with pytest.raises(OracleError):
        o.prefetch(np.array([10]), np.array([0, 1]))
    with pytest.raises(OracleError):
        o.prefetch(np.array([1, 2]), np.array([0, 2, 1, 2]), batch=3)
    with pytest.raises(OracleError):
        o.forward()
    o.prefetch(np.array([1]), np.array([0, 1]))
    with pytest.raises(OracleError):
        o.backward_update(np.zeros((1, 4), dtype=np.float32), 0.1, 1e-8)


def test_row_peak_bookkeeping():
    """The tests' error bars use the largest magnitude a row has held since the run began.  One row, one
    element driven down, up and down again by hand: w0 = 0.5; gradient +1 once (the row drops to 0, so the peak
    is the value it had before the update), -1 three times, then +1 many times."""
    W = [np.array([[0.5], [0.25]], dtype=np.float32)]
    M = [np.zeros(2, dtype=np.float32)]
    o = Oracle(W, M, [0], ways=1)
    assert o.row_peak(0).tolist() == [0.0, 0.0]
    w, m, lr, top = 0.5, 0.0, 0.5, 0.5
    for k in range(14):
        g = -1.0 if 1 <= k < 4 else 1.0
        o.prefetch(np.array([0]), np.array([0, 1]))
        o.forward()
        o.backward_update(np.array([[g]], dtype=np.float32), lr, 0.0)
        m += g * g
        w = float(np.float32(w - lr * g / np.sqrt(m)))
        top = max(top, abs(w))
        assert o.row_peak(0)[0] == pytest.approx(top, rel=1e-6) and o.row_peak(0)[1] == 0.0
    assert abs(w) < top  # the peak lies in the past
    assert W[0][0, 0] == pytest.approx(w, rel=1e-6)
