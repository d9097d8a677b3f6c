"""Pins of the oracle's LFU policy (the other replacement policy the paper tried,
Section 5.5.2) against things other than itself: an independent per-set list model, a
textbook LFU with least-recently-used tie-break for batches of one lookup, a hand-worked
example, and the properties that tell LFU from LRU.  CPU only."""
import numpy as np
import pytest

from oracle import Oracle, OracleError
from test_oracle_pins import RNG, make_tables, random_batch


class LfuListModel:
    """Per set an explicit list of [way, tag, ts, count]; a batch first credits the hits
    (count += lookups of the row, ts = k), then gives the misses, in ascending row order,
    the entries older than k in order of (count, ts, way)."""

    def __init__(self, sets, ways):
        self.sets, self.ways = sets, ways
        self.s = [[[w, -1, -1, 0] for w in range(ways)] for _ in range(sets)]

    def batch(self, rows, k):
        mult = {}
        for r in rows:
            mult[r] = mult.get(r, 0) + 1
        hits, ins, byp = [], [], []
        for s in range(self.sets):
            q = sorted(r for r in mult if r % self.sets == s)
            ent = self.s[s]
            where = {e[1]: e for e in ent if e[1] >= 0}
            miss = []
            for r in q:
                if r in where:
                    where[r][2] = k
                    where[r][3] += mult[r]
                    hits.append(r)
                else:
                    miss.append(r)
            order = sorted((e for e in ent if e[2] < k), key=lambda e: (e[3], e[2], e[0]))
            for j, r in enumerate(miss):
                if j < len(order):
                    e = order[j]
                    ins.append((r, s * self.ways + e[0], e[1]))
                    e[1], e[2], e[3] = r, k, mult[r]
                else:
                    byp.append(r)
        return sorted(hits), sorted(ins), sorted(byp)

    def state(self):
        flat = [e for s in self.s for e in sorted(s)]
        return (np.array([e[1] for e in flat], dtype=np.int64), np.array([e[2] for e in flat], dtype=np.int32),
                np.array([e[3] for e in flat], dtype=np.int32))


@pytest.mark.parametrize("sets,ways,H,n", [(1, 4, 40, 6), (3, 2, 50, 9), (5, 8, 200, 60), (7, 3, 64, 40), (2, 64, 4000, 150)])
def test_lfu_state_matches_list_model(sets, ways, H, n):
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [sets * ways], ways=ways, policy="lfu")
    model = LfuListModel(sets, ways)
    g = RNG(sets * 100 + ways + 1)
    for k in range(1, 60):
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
        mt, mts, mf = model.state()
        assert np.array_equal(tags, mt) and np.array_equal(ts, mts) and np.array_equal(o.cache_freq(0), mf)


def test_single_lookup_batches_are_textbook_lfu():
    """One lookup per batch and one set: the classic LFU -- a dictionary row -> (uses, last
    use); on a miss with a full cache the row with the fewest uses leaves, the least
    recently used among those."""
    ways, H = 5, 40
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [ways], ways=ways, policy="lfu")
    book = {}
    g = RNG(7)
    for k in range(1, 600):
        r = int(g.integers(0, H) if k % 4 == 0 else g.integers(0, 9))
        o.prefetch(np.array([r]), np.array([0, 1]))
        st = o.stats()[0]
        if r in book:
            assert st["hits"] == 1
            book[r] = (book[r][0] + 1, k)
        else:
            assert st["inserts"] == 1 and st["bypasses"] == 0
            _, _, _, old = o.events("insert")
            if len(book) == ways:
                out = min(book, key=lambda x: book[x])
                assert old[0] == out
                del book[out]
            else:
                assert old[0] == -1
            book[r] = (1, k)
        tags, ts = o.cache_state(0)
        f = o.cache_freq(0)
        assert {int(t): (int(c), int(s)) for t, s, c in zip(tags, ts, f) if t >= 0} == book


def test_hand_worked_example():
    # one set, 3 ways.  k=1: rows 4,4,4,9,2 -> inserted in ascending order 2,4,9 into ways 0,1,2
    # with counts 1,3,1.  k=2: row 9 twice -> count 3.  k=3: row 7 misses: candidates are all three
    # ways (none stamped 3); counts 1,3,3 -> way 0 (row 2) leaves.  k=4: row 5 misses: counts
    # (7:1, 4:3, 9:3) -> row 7 leaves although it is the most recent one (LRU would take row 4).
    W, M = make_tables([16], [4], [np.float32])
    o = Oracle(W, M, [3], ways=3, policy="lfu")
    o.prefetch(np.array([4, 4, 4, 9, 2]), np.array([0, 5]))
    assert o.cache_state(0)[0].tolist() == [2, 4, 9] and o.cache_freq(0).tolist() == [1, 3, 1]
    o.prefetch(np.array([9, 9]), np.array([0, 2]))
    assert o.cache_freq(0).tolist() == [1, 3, 3] and o.cache_state(0)[1].tolist() == [1, 1, 2]
    o.prefetch(np.array([7]), np.array([0, 1]))
    assert o.events("insert")[3].tolist() == [2]
    assert o.cache_state(0)[0].tolist() == [7, 4, 9] and o.cache_freq(0).tolist() == [1, 3, 3]
    o.prefetch(np.array([5]), np.array([0, 1]))
    assert o.events("insert")[3].tolist() == [7]
    assert o.cache_state(0)[0].tolist() == [5, 4, 9] and o.cache_state(0)[1].tolist() == [4, 1, 2]
    # the same sequence under LRU evicts row 4 at k=4
    o2 = Oracle(*make_tables([16], [4], [np.float32]), [3], ways=3, policy="lru")
    for b in ([4, 4, 4, 9, 2], [9, 9], [7], [5]):
        o2.prefetch(np.array(b), np.array([0, len(b)]))
    assert o2.events("insert")[3].tolist() == [4]


def test_frequent_row_survives_a_scan_under_lfu_only():
    # a row used 10 times, then a scan of one-time rows longer than the set: LFU keeps it, LRU drops it
    for policy, kept in (("lfu", True), ("lru", False)):
        W, M = make_tables([100], [4], [np.float32])
        o = Oracle(W, M, [4], ways=4, policy=policy)
        for _ in range(10):
            o.prefetch(np.array([0]), np.array([0, 1]))
        for r in range(1, 12):
            o.prefetch(np.array([r]), np.array([0, 1]))
        assert (0 in o.cache_state(0)[0].tolist()) == kept


def test_locked_ways_and_bypass_are_the_same_as_lru():
    # a batch with more distinct rows than ways: the lowest rows are inserted, the rest bypass
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [2], ways=2, policy="lfu")
    o.prefetch(np.array([7, 1, 5, 3, 1]), np.array([0, 5]))
    assert o.events("insert")[1].tolist() == [1, 3] and o.events("bypass")[1].tolist() == [5, 7]
    assert o.cache_freq(0).tolist() == [2, 1]
    # the next batch hits row 3 (locked), and row 9 must take row 1's way although row 1 has the higher count
    o.prefetch(np.array([3, 9]), np.array([0, 2]))
    assert o.cache_state(0)[0].tolist() == [9, 3] and o.cache_freq(0).tolist() == [1, 2]


def test_values_do_not_depend_on_the_policy():
    rows, dims = [300, 50], [8, 4]
    res = {}
    for policy in ("lru", "lfu"):
        W, M = make_tables(rows, dims, [np.float32, np.float16], seed=3)
        o = Oracle(W, M, [32, 8], ways=4, policy=policy)
        outs = []
        for k in range(12):
            idx, off = random_batch(rows, 6, 5, seed=100 + k)
            o.prefetch(idx, off)
            outs.append(o.forward().copy())
            go = RNG(k).standard_normal((6, sum(dims))).astype(np.float32)
            o.backward_update(go, 0.05, 1e-8)
            last = o.stats()[0]
            assert last["hits"] + last["inserts"] + last["bypasses"] == last["uniques"]
        o.flush()
        res[policy] = (outs, [w.copy() for w in W], [m.copy() for m in M], o.stats()[1])
    for a, b in zip(res["lru"][0], res["lfu"][0]):
        assert np.array_equal(a, b)
    for t in range(2):
        assert np.array_equal(res["lru"][1][t], res["lfu"][1][t]) and np.array_equal(res["lru"][2][t], res["lfu"][2][t])
    assert res["lru"][3] != res["lfu"][3]  # the two policies do differ in what they keep


def test_full_capacity_never_evicts_under_lfu():
    H, ways = 64, 4
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [H], ways=ways, policy="lfu")
    g = RNG(5)
    seen = set()
    for k in range(30):
        rows = g.integers(0, H, size=20)
        o.prefetch(rows, np.array([0, 20]))
        st = o.stats()[0]
        new = set(rows.tolist()) - seen
        assert st["inserts"] == len(new) and st["evictions"] == 0 and st["bypasses"] == 0
        seen |= set(rows.tolist())
    # counts are the total lookups of every row
    tags, f = o.cache_state(0)[0], o.cache_freq(0)
    assert f.sum() == 30 * 20 and (f[tags < 0] == 0).all()


def test_policy_is_fixed_before_the_first_batch():
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [4], ways=2)
    o.prefetch(np.array([1]), np.array([0, 1]))
    from oracle import lib
    assert lib().orc_set_policy(o.h, 1) != 0
    assert lib().orc_set_policy(o.h, 7) != 0
    with pytest.raises(KeyError):
        Oracle(W, M, [4], ways=2, policy="fifo")


def test_lfu_count_saturates_at_int32_max():
    """The per-entry lookup count stops at INT32_MAX: it neither wraps to a negative number nor grows on in a
    wider type.  Hand-worked on one set of two ways (counts are put near the limit through the oracle's test
    hook; reaching them by lookups would take two billion of them):
      batch 1: row 0 three times, row 1 twice           -> ways (0, 1) hold rows (0, 1), counts (3, 2)
      counts set to (INT32_MAX - 2, INT32_MAX - 1)
      batch 2: row 0 five times, row 1 once             -> both hit; exact sums would be INT32_MAX + 3 and INT32_MAX:
                                                           both counts must read INT32_MAX
      batch 3: row 2 once (a miss)                      -> candidates tie on count and on timestamp (2, 2), so the
                                                           lowest way goes: row 0 leaves way 0.  A wider counter would
                                                           keep row 0 (larger count) and evict row 1 from way 1; a
                                                           wrapped one would read negative in the export."""
    big = np.iinfo(np.int32).max
    W, M = make_tables([10], [4], [np.float32])
    o = Oracle(W, M, [2], ways=2, policy="lfu")

    def batch(rows):
        idx = np.array(rows, dtype=np.int64)
        o.prefetch(idx, np.array([0, len(rows)], dtype=np.int64))
        o.forward()
        o.backward_update(np.zeros((1, 4), dtype=np.float32), 0.01, 1e-8)

    batch([0, 0, 0, 1, 1])
    assert o.cache_state(0)[0].tolist() == [0, 1] and o.cache_freq(0).tolist() == [3, 2]
    o.set_cache_freq(0, np.array([big - 2, big - 1], dtype=np.int32))
    batch([0, 0, 0, 0, 0, 1])
    assert o.cache_freq(0).tolist() == [big, big]
    batch([2])
    tags, ts = o.cache_state(0)
    assert tags.tolist() == [2, 1] and ts.tolist() == [3, 2]
    assert o.cache_freq(0).tolist() == [1, big]
    _, rows, slots, old = o.events("insert")
    assert (rows.tolist(), slots.tolist(), old.tolist()) == ([2], [0], [0])
    o.close()
