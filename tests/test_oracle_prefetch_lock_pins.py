"""Pins of the oracle's optional lock over the ways stamped by the `L` batches before the current one (the rule
of Section 5.7 for a pipeline that fetches L batches ahead: rows fetched for a batch stay in the cache until that
batch has trained), against things other than the oracle: an independent list model written here, the invariant
itself checked from the index stream, a hand-worked case, the textbook LRU stack for one-lookup batches, and the
uncached trainer for the values.  CPU only."""
import numpy as np
import pytest

from oracle import Oracle
from test_oracle_pins import RNG, make_tables, random_batch


class LockedListModel:
    """Per set a list of [way, tag, ts]: hits are stamped, then the misses (ascending) take the entries in order
    of (ts, way) among the free ones and those with ts < k - lock; the rest of the misses bypass."""

    def __init__(self, sets, ways, lock):
        self.sets, self.ways, self.lock = sets, ways, lock
        self.s = [[[w, -1, -1] for w in range(ways)] for _ in range(sets)]

    def batch(self, rows, k):
        hits, ins, byp = [], [], []
        for s in range(self.sets):
            q = sorted(r for r in set(rows) if r % self.sets == s)
            ent = self.s[s]
            present = {e[1]: e for e in ent if e[1] >= 0}
            miss = []
            for r in q:
                if r in present:
                    present[r][2] = k
                    hits.append(r)
                else:
                    miss.append(r)
            free = sorted((e for e in ent if e[1] < 0 or e[2] < k - self.lock), key=lambda e: (e[2], e[0]))
            for j, r in enumerate(miss):
                if j < len(free):
                    e = free[j]
                    ins.append((r, s * self.ways + e[0], e[1]))
                    e[1], e[2] = r, k
                else:
                    byp.append(r)
        return sorted(hits), sorted(ins), sorted(byp)

    def state(self):
        return (np.array([e[1] for s in self.s for e in sorted(s)], dtype=np.int64),
                np.array([e[2] for s in self.s for e in sorted(s)], dtype=np.int32))


@pytest.mark.parametrize("lock", [1, 2, 3])
@pytest.mark.parametrize("sets,ways,H,n", [(1, 4, 40, 5), (3, 2, 50, 4), (5, 8, 200, 30), (2, 64, 4000, 90)])
def test_locked_cache_matches_list_model_and_keeps_the_invariant(sets, ways, H, n, lock):
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [sets * ways], ways=ways, prefetch_lock=lock)
    model = LockedListModel(sets, ways, lock)
    g = RNG(sets * 1000 + ways * 10 + lock)
    last_seen = {}  # row -> last batch that looked it up
    evictions = 0
    for k in range(1, 50):
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
        # Section 5.7 at this depth: no row that one of the batches k - lock .. k looked up is evicted by batch k
        for old in iold.tolist():
            if old >= 0:
                evictions += 1
                assert last_seen[old] < k - lock
        # ... so every cached row of those batches is still resident
        bypassed = set(byp)
        for r, seen in last_seen.items():
            if seen >= k - lock and r in set(tags.tolist()):
                assert ts[tags.tolist().index(r)] >= seen
        for r in set(rows.tolist()) - bypassed:
            last_seen[r] = k
        for r in bypassed:
            last_seen.setdefault(r, -1)
    assert evictions > 0 or ways >= 64


def test_hand_worked_case():
    """One set of two ways, lock 1.  Batch 1 {1, 2}: both inserted.  Batch 2 {3}: both ways were stamped by the
    batch before and are locked, so 3 bypasses (without the lock it would take way 0).  Batch 3 {4}: the ways
    carry timestamp 1 < 3 - 1, the lower way goes: row 1 is evicted."""
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [2], ways=2, prefetch_lock=1)
    o.prefetch(np.array([1, 2]), np.array([0, 2]))
    o.prefetch(np.array([3]), np.array([0, 1]))
    assert o.events("bypass")[1].tolist() == [3] and o.events("insert")[1].size == 0
    o.prefetch(np.array([4]), np.array([0, 1]))
    _, ir, isl, iold = o.events("insert")
    assert (ir.tolist(), isl.tolist(), iold.tolist()) == ([4], [0], [1])
    tags, ts = o.cache_state(0)
    assert tags.tolist() == [4, 2] and ts.tolist() == [3, 1]
    plain = Oracle(*make_tables([10], [4], [np.float32]), [2], ways=2)
    plain.prefetch(np.array([1, 2]), np.array([0, 2]))
    plain.prefetch(np.array([3]), np.array([0, 1]))
    assert plain.events("insert")[1].tolist() == [3] and plain.events("bypass")[1].size == 0


@pytest.mark.parametrize("lock", [1, 3])
def test_one_lookup_batches_with_more_ways_than_locked_batches_are_plain_lru(lock):
    """A batch of one lookup stamps one way, so the `lock` batches before the current one hold at most `lock`
    ways of a set; with more ways than that the least recently used way is never one of them, and the cache is
    the textbook LRU stack, lock or no lock."""
    H, sets, ways = 60, 3, lock + 1
    g = RNG(5 + lock)
    a = Oracle(*make_tables([H], [4], [np.float32]), [sets * ways], ways=ways, prefetch_lock=lock)
    b = Oracle(*make_tables([H], [4], [np.float32]), [sets * ways], ways=ways)
    mtf = [[] for _ in range(sets)]
    for k in range(1, 300):
        r = int(g.integers(0, H))
        for o in (a, b):
            o.prefetch(np.array([r]), np.array([0, 1]))
        lst = mtf[r % sets]
        if r in lst:
            lst.remove(r)
        lst.insert(0, r)
        del lst[ways:]
        ta, tsa = a.cache_state(0)
        tb, tsb = b.cache_state(0)
        assert np.array_equal(ta, tb) and np.array_equal(tsa, tsb)
        for s in range(sets):
            assert set(ta[s * ways:(s + 1) * ways].tolist()) - {-1} == set(mtf[s])


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_values_do_not_depend_on_the_lock(dtype):
    """The cache is transparent: pooled outputs and, after a flush, every row and accumulator equal those of a
    trainer without a cache (zero slots), whatever the lock; the lock only turns inserts into bypasses."""
    rows, dims = [300, 120], [8, 16]
    runs = []
    for slots, lock in (([0, 0], 0), ([32, 16], 0), ([32, 16], 2)):
        W, M = make_tables(rows, dims, [dtype, dtype], seed=3)
        o = Oracle(W, M, slots, ways=4, prefetch_lock=lock)
        outs, byp = [], 0
        for step in range(12):
            idx, off = random_batch(rows, 6, 5, seed=100 + step)
            o.prefetch(idx, off)
            outs.append(o.forward().copy())
            go = RNG(200 + step).standard_normal((6, sum(dims))).astype(np.float32)
            o.backward_update(go, 0.05, 1e-8)
            byp += o.stats()[0]["bypasses"]
        o.flush()
        runs.append((outs, [w.copy() for w in W], [m.copy() for m in M], byp))
    for outs, Ws, Ms, _ in runs[1:]:
        assert all(np.array_equal(x, y) for x, y in zip(outs, runs[0][0]))
        assert all(np.array_equal(x, y) for x, y in zip(Ws, runs[0][1]))
        assert all(np.array_equal(x, y) for x, y in zip(Ms, runs[0][2]))
    assert runs[2][3] >= runs[1][3]
