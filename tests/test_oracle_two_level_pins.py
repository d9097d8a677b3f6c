"""Pins of the oracle's two-level exclusive cache (Section 5.3, 5.5.4) against things other
than itself: the LRU stack a two-level exclusive hierarchy must be for batches of one
lookup, an independent dictionary model, a hand-worked example, and the invariants
(exclusivity, values independent of the cache sizes, conservation of the counters)."""
import numpy as np
import pytest

from oracle import Oracle
from test_oracle_pins import RNG, make_tables, random_batch


def contents(tags):
    return set(int(t) for t in tags if t >= 0)


def test_single_lookup_batches_form_one_lru_stack():
    """One set per level, one lookup per batch: first level = the W most recently used
    rows, second level = the next W -- together a move-to-front list of 2 W rows."""
    ways, H = 4, 40
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [ways], ways=ways, second_level_slots=[ways])
    stack = []
    g = RNG(3)
    for k in range(1, 500):
        r = int(g.integers(0, H) if k % 3 == 0 else g.integers(0, 11))
        o.prefetch(np.array([r]), np.array([0, 1]))
        st, l2 = o.stats()[0], o.second_level_stats()[0]
        if r in stack[:ways]:
            assert st["hits"] == 1 and l2["hits"] == 0
        elif r in stack:
            assert st["inserts"] == 1 and l2["hits"] == 1
        else:
            assert st["inserts"] == 1 and l2["hits"] == 0
            if len(stack) == 2 * ways:
                assert l2["evictions"] == 1
        if r in stack:
            stack.remove(r)
        stack.insert(0, r)
        del stack[2 * ways:]
        assert contents(o.cache_state(0)[0]) == set(stack[:ways])
        assert contents(o.second_level_state(0)[0]) == set(stack[ways:])


class TwoLevelModel:
    """Dictionaries instead of arrays: level -> set -> {way: [row, ts]}."""

    def __init__(self, s1, s2, ways):
        self.s1, self.s2, self.w = s1, s2, ways
        self.l1 = [dict() for _ in range(s1)]
        self.l2 = [dict() for _ in range(s2)]

    @staticmethod
    def _victim_way(entries, ways, before):
        """way whose entry is free or stamped earlier than `before`: oldest first, lowest way among equals"""
        cand = [(entries[w][1] if w in entries else -1, w) for w in range(ways) if w not in entries or entries[w][1] < before]
        return min(cand)[1] if cand else None

    def batch(self, rows, k):
        uniq = sorted(set(rows))
        missed, victims, inserted = [], [], set()
        for s in range(self.s1):
            q = [r for r in uniq if r % self.s1 == s]
            ent = self.l1[s]
            here = {v[0]: w for w, v in ent.items()}
            for r in q:
                if r in here:
                    ent[here[r]][1] = k
            for r in q:
                if r in here:
                    continue
                missed.append(r)
                w = self._victim_way(ent, self.w, k)
                if w is None:
                    continue
                if w in ent:
                    victims.append(ent[w][0])
                ent[w] = [r, k]
                inserted.add(r)
        hits2 = 0
        for r in sorted(missed):
            ent = self.l2[r % self.s2]
            w = next((w for w, v in ent.items() if v[0] == r), None)
            if w is None:
                continue
            hits2 += 1
            if r in inserted:
                del ent[w]
            else:
                ent[w][1] = k
        ev2 = byp2 = 0
        for v in sorted(victims):
            ent = self.l2[v % self.s2]
            w = self._victim_way(ent, self.w, k - 1)  # entries of this batch and the one before stay
            if w is None:
                byp2 += 1
                continue
            ev2 += w in ent
            ent[w] = [v, k]
        return hits2, len(victims) - byp2, ev2, byp2

    @staticmethod
    def _flat(level, ways):
        tags = [level[s][w][0] if w in level[s] else -1 for s in range(len(level)) for w in range(ways)]
        ts = [level[s][w][1] if w in level[s] else -1 for s in range(len(level)) for w in range(ways)]
        return tags, ts


@pytest.mark.parametrize("s1,s2,ways,H,n", [(1, 1, 4, 60, 8), (2, 6, 3, 90, 14), (3, 12, 8, 400, 70), (5, 7, 2, 64, 30),
                                            (2, 4, 64, 4000, 200)])
def test_state_matches_dictionary_model(s1, s2, ways, H, n):
    W, M = make_tables([H], [4], [np.float32])
    o = Oracle(W, M, [s1 * ways], ways=ways, second_level_slots=[s2 * ways])
    model = TwoLevelModel(s1, s2, ways)
    g = RNG(s1 * 1000 + s2 * 10 + ways)
    for k in range(1, 60):
        m = int(g.integers(1, n + 1))
        rows = np.minimum(g.pareto(0.6, size=m).astype(np.int64) * 3 + g.integers(0, 3, size=m), H - 1)
        o.prefetch(rows, np.array([0, m]))
        h2, d2, e2, b2 = model.batch(rows.tolist(), k)
        assert o.second_level_stats()[0] == {"hits": h2, "demotions": d2, "evictions": e2, "bypasses": b2}
        t1, ts1 = model._flat(model.l1, ways)
        t2, ts2 = model._flat(model.l2, ways)
        assert o.cache_state(0)[0].tolist() == t1 and o.cache_state(0)[1].tolist() == ts1
        assert o.second_level_state(0)[0].tolist() == t2 and o.second_level_state(0)[1].tolist() == ts2
        # exclusive: no row in both levels
        assert not (contents(o.cache_state(0)[0]) & contents(o.second_level_state(0)[0]))
        st = o.stats()[0]
        assert d2 + b2 == st["evictions"] and h2 <= st["inserts"] + st["bypasses"]


def test_hand_worked_example():
    # first level: one set of 2 ways; second level: one set of 2 ways.
    W, M = make_tables([20], [4], [np.float32])
    o = Oracle(W, M, [2], ways=2, second_level_slots=[2])
    o.prefetch(np.array([1, 2]), np.array([0, 2]))          # k=1: L1 = [1, 2]
    o.prefetch(np.array([3]), np.array([0, 1]))             # k=2: 3 takes way 0 (row 1, older ts tie -> lowest way); 1 -> L2 way 0
    assert o.cache_state(0)[0].tolist() == [3, 2] and o.second_level_state(0)[0].tolist() == [1, -1]
    o.prefetch(np.array([4]), np.array([0, 1]))             # k=3: 4 takes way 1 (row 2, ts 1); 2 -> L2 way 1
    assert o.cache_state(0)[0].tolist() == [3, 4] and o.second_level_state(0)[0].tolist() == [1, 2]
    assert o.second_level_state(0)[1].tolist() == [2, 3]
    o.prefetch(np.array([1]), np.array([0, 1]))             # k=4: 1 found in L2 -> moves up into way 0 (row 3, ts 2);
    #                                                         its L2 way is free again and takes row 3
    assert o.cache_state(0)[0].tolist() == [1, 4] and o.second_level_state(0)[0].tolist() == [3, 2]
    assert o.second_level_stats()[0] == {"hits": 1, "demotions": 1, "evictions": 0, "bypasses": 0}
    o.prefetch(np.array([5]), np.array([0, 1]))             # k=5: 5 takes way 1 (row 4, ts 3); 4 -> L2: oldest is row 2 (ts 3)
    assert o.cache_state(0)[0].tolist() == [1, 5] and o.second_level_state(0)[0].tolist() == [3, 4]
    assert o.second_level_stats()[0] == {"hits": 0, "demotions": 1, "evictions": 1, "bypasses": 0}
    # three distinct rows in one batch: the third bypasses the first level; it is in L2 and is used in place
    o.prefetch(np.array([3, 6, 7]), np.array([0, 3]))       # k=6: 3 (L2 hit, moves up), 6 inserted, 7 bypasses
    assert o.cache_state(0)[0].tolist() == [3, 6]
    assert o.events("bypass")[1].tolist() == [7]
    # victims 1 and 5 move down in that order: row 1 takes the way row 3 left; row 4 entered at k=5, the batch
    # before, so its way stays and row 5 goes straight to the lower tier
    assert o.second_level_state(0)[0].tolist() == [1, 4] and o.second_level_state(0)[1].tolist() == [6, 5]
    assert o.second_level_stats()[0] == {"hits": 1, "demotions": 1, "evictions": 0, "bypasses": 1}


def uncached_reference(rows, dims, dt, steps, seed):
    W, M = make_tables(rows, dims, [dt] * len(rows), seed=seed)
    o = Oracle(W, M, [0] * len(rows), ways=4)
    outs = []
    for s in range(steps):
        idx, off = random_batch(rows, 12, 5, seed=300 + s)
        o.prefetch(idx, off)
        outs.append(o.forward().copy())
        o.backward_update(RNG(400 + s).standard_normal((12, sum(dims))).astype(np.float32), 0.05, 1e-8)
    return outs, W, M


@pytest.mark.parametrize("dt", [np.float32, np.float16])
@pytest.mark.parametrize("slots,slots2", [([16, 8], [32, 8]), ([4, 4], [64, 0]), ([0, 8], [16, 16]), ([64, 64], [4, 4])])
def test_values_do_not_depend_on_the_hierarchy(dt, slots, slots2):
    rows, dims, steps = [300, 70], [8, 4], 10
    ref_out, ref_W, ref_M = uncached_reference(rows, dims, dt, steps, seed=5)
    W, M = make_tables(rows, dims, [dt] * 2, seed=5)
    o = Oracle(W, M, slots, ways=4, second_level_slots=slots2)
    for s in range(steps):
        idx, off = random_batch(rows, 12, 5, seed=300 + s)
        o.prefetch(idx, off)
        assert np.array_equal(o.forward(), ref_out[s])
        o.backward_update(RNG(400 + s).standard_normal((12, sum(dims))).astype(np.float32), 0.05, 1e-8)
        # a row read wherever it lives has the value of the uncached trainer only after flush; before that the
        # lower tier may be stale, but never the copy the hierarchy points to (checked through the next forward)
    o.flush()
    for t in range(2):
        assert np.array_equal(W[t], ref_W[t]) and np.array_equal(M[t], ref_M[t])
    tot2 = o.second_level_stats()[1]
    if slots == [16, 8]:
        assert tot2["demotions"] > 0 and tot2["hits"] > 0 and tot2["evictions"] > 0


def test_no_second_level_is_the_one_level_cache():
    rows, dims = [200], [8]
    res = []
    for s2 in (None, [0]):
        W, M = make_tables(rows, dims, [np.float32], seed=2)
        o = Oracle(W, M, [16], ways=4, second_level_slots=s2)
        for k in range(8):
            idx, off = random_batch(rows, 6, 5, seed=50 + k)
            o.prefetch(idx, off)
            o.forward()
            o.backward_update(RNG(k).standard_normal((6, 8)).astype(np.float32), 0.05, 1e-8)
        res.append((o.cache_state(0)[0].copy(), o.cache_state(0)[1].copy(), o.stats()[1], W[0].copy()))
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])
    assert res[0][2] == res[1][2] and np.array_equal(res[0][3], res[1][3])


def test_lower_tier_is_stale_until_flush_and_second_level_holds_trained_rows():
    # a row trained in the first level and then pushed down must carry its trained value in the second level
    W, M = make_tables([10], [4], [np.float32], seed=1, std=1.0)
    W0 = W[0].copy()
    o = Oracle(W, M, [1], ways=1, second_level_slots=[4])
    o.prefetch(np.array([3]), np.array([0, 1]))
    o.forward()
    o.backward_update(np.ones((1, 4), dtype=np.float32), 0.5, 1e-8)
    o.prefetch(np.array([4]), np.array([0, 1]))  # row 3 moves down
    o.forward()
    o.backward_update(np.zeros((1, 4), dtype=np.float32), 0.5, 1e-8)
    assert np.array_equal(W[0][3], W0[3])  # lower tier still has the old value
    w3, m3 = o.read_row(0, 3)
    np.testing.assert_allclose(w3, W0[3] - 0.5 * 1.0 / (1.0 + 1e-8), rtol=1e-6)
    assert m3 == pytest.approx(1.0)
    o.flush()
    np.testing.assert_allclose(W[0][3], w3, rtol=1e-7)


def test_victim_goes_straight_down_when_its_second_level_set_is_locked():
    # one way per level.  k=1: row 1 in L1.  k=2: row 2 in L1 (trained), row 1 in L2.  k=3: batch {0, 1}: row 0 is
    # inserted (row 2 leaves L1), row 1 bypasses L1, is found in L2 and stamped 3 -- so L2's only way is locked and
    # row 2, with its trained value and accumulator, must land in the lower tier at once.
    W, M = make_tables([10], [4], [np.float32], seed=1, std=1.0)
    W0 = W[0].copy()
    o = Oracle(W, M, [1], ways=1, second_level_slots=[1])
    for r, g in ((1, 0.0), (2, 1.0)):
        o.prefetch(np.array([r]), np.array([0, 1]))
        o.forward()
        o.backward_update(np.full((1, 4), g, dtype=np.float32), 0.5, 1e-8)
    assert np.array_equal(W[0][2], W0[2])
    o.prefetch(np.array([0, 1]), np.array([0, 2]))
    assert o.second_level_stats()[0] == {"hits": 1, "demotions": 0, "evictions": 0, "bypasses": 1}
    assert o.cache_state(0)[0].tolist() == [0] and o.second_level_state(0)[0].tolist() == [1]
    np.testing.assert_allclose(W[0][2], W0[2] - 0.5 / (1.0 + 1e-8), rtol=1e-6)
    assert M[0][2] == pytest.approx(1.0)


def test_counters_are_per_batch_also_for_a_table_without_lookups():
    # two tables, each against its own dictionary model; the second one sits out every other batch, and a
    # batch's second-level counters must then be those of the first table alone
    ways, H = 2, 40
    W, M = make_tables([H, H], [4, 4], [np.float32] * 2)
    o = Oracle(W, M, [2 * ways] * 2, ways=ways, second_level_slots=[4 * ways] * 2)
    models = [TwoLevelModel(2, 4, ways), TwoLevelModel(2, 4, ways)]
    g = RNG(77)
    total = np.zeros(4, dtype=np.int64)
    idle_after_busy = 0
    for k in range(1, 80):
        rows = [g.integers(0, H, size=int(g.integers(3, 9))), g.integers(0, H, size=0 if k % 2 else int(g.integers(3, 9)))]
        o.prefetch(np.concatenate(rows), np.array([0, len(rows[0]), len(rows[0]) + len(rows[1])]))
        per = [m.batch(r.tolist(), k) if len(r) else (0, 0, 0, 0) for m, r in zip(models, rows)]
        want = np.array(per).sum(axis=0)
        total += want
        last, tot = o.second_level_stats()
        assert list(last.values()) == want.tolist() and list(tot.values()) == total.tolist()
        idle_after_busy += int(len(rows[1]) == 0 and k > 1 and prev_busy > 0)
        prev_busy = sum(per[1])
    assert idle_after_busy > 10  # the case that matters: an idle batch right after one that moved rows


def test_two_batch_lock_of_the_second_level_changes_nothing_but_its_occupancy():
    """The library's second level does not replace entries stamped by the current batch OR the one before (its data
    moves trail its decisions by a batch); a sequential model has no data in flight and would lock the current
    batch's entries only (the plain reading of the rule of Section 5.7).  Both rules run side by side on the same
    stream: pooled outputs, every row and accumulator, the first level's tags and timestamps and the first level's
    counters must be identical batch for batch -- the first level never looks at the second -- and only the
    second level's contents and counters may differ.  The cost of the extra lock is then a number: rows found in
    the second level under either rule (printed; the two-batch lock keeps recently demoted rows longer and lets
    more victims pass the second level by)."""
    rows, dims = [3000, 800], [8, 4]
    ways = 4
    slots1, slots2 = [ways * 12, ways * 5], [ways * 12, ways * 5]  # small second level: sets fill up within two batches
    runs = []
    for lock in (1, 2):
        W, M = make_tables(rows, dims, [np.float32, np.float16], seed=5)
        o = Oracle(W, M, slots1, ways=ways, second_level_slots=slots2, second_level_lock=lock)
        trace, found, passed_by = [], 0, 0
        for k in range(1, 41):
            idx, off = random_batch(rows, 24, 5, seed=100 + k, skew=k % 3 != 0)
            o.prefetch(idx, off)
            out = o.forward().copy()
            go = RNG(k).standard_normal((24, sum(dims))).astype(np.float32)
            o.backward_update(go, 0.05, 1e-8)
            l2 = o.second_level_stats()[0]
            found += l2["hits"]
            passed_by += l2["bypasses"]
            trace.append((out, [tuple(a.copy() for a in o.cache_state(t)) for t in range(2)], o.stats()[0]))
        l2_state = [tuple(a.copy() for a in o.second_level_state(t)) for t in range(2)]
        o.flush()
        o.close()
        runs.append((trace, W, M, l2_state, found, passed_by))
    a, b = runs
    for k, ((out_a, st_a, cnt_a), (out_b, st_b, cnt_b)) in enumerate(zip(a[0], b[0])):
        assert np.array_equal(out_a, out_b), f"pooled output of batch {k + 1} depends on the second level's rule"
        assert cnt_a == cnt_b
        for (ta, sa), (tb, sb) in zip(st_a, st_b):
            assert np.array_equal(ta, tb) and np.array_equal(sa, sb)
    for t in range(2):
        assert np.array_equal(a[1][t], b[1][t]) and np.array_equal(a[2][t], b[2][t])
    assert any(not np.array_equal(x[0], y[0]) for x, y in zip(a[3], b[3])), "the two rules never differed: the case is too easy"
    assert a[5] <= b[5]  # the wider lock can only make more victims pass the second level by ... on this stream
    print(f"second-level hits: lock of 1 batch {a[4]}, of 2 batches {b[4]}; victims passing it by: {a[5]} / {b[5]}")
