"""Shared driver of the GPU parity tests: runs the CPU oracle and the HIP library on
the same seeded inputs and compares them step by step.

Bars (written here once, used by every parity test):
  - cache state (tags, timestamps, per-entry lookup counts), per-batch counters and the hit / insert / bypass
    event sets: bit-exact;
  - floating point, per vector v against the oracle's r (a pooled bag slice, an updated
    row):  max_d |v - r| <= tol * max(max_d |r|, floor), tol = 1e-5 for fp32 storage and
    2e-3 for fp16 storage (fp32 accumulation); the accumulator m always with 1e-5 (floor M_FLOOR).
    This plain bar is applied to every vector first.  Only for fp16 storage under max pooling a vector
    that misses it is then held against the wider scale max(max_d |r|, peak, floor), `peak` being the
    largest magnitude the row (for a pooled slice: any row of the bag) has held since the run began, kept
    by the oracle: a rounding to binary16 that fell differently on the two sides while a row was large
    stays in it as an absolute difference when the row shrinks (one fp16 ulp taken at 0.5 is four ulps at
    0.15), and max pooling's sparse gradients make rows grow to 1 and shrink again within a few steps.
    Every vector that needed the wider scale is counted (`Tally`); run_parity returns the count and the
    worst ratio to the plain bar, and asserts that the count is 0 for fp32 storage and for sum and mean
    pooling;
  - max pooling, who supplied each maximum: equal, except where two different rows' values lie within
    the floating-point bar of each other in the oracle (stored values agree only to that bar once rows
    have been updated, so either row may hold the larger one).  Such a choice is checked to be a valid
    one; the two sides train different rows from there on, so values are no longer compared after it
    (cache state, counters and events still are, to the end) and the step is reported as 'parted_at'.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import Oracle
from paper_2305_01515_amd import synth

TOL = {synth.FP32: 1e-5, synth.FP16: 2e-3}
# Accumulators: |m - ref| <= 1e-5 * max(ref, M_FLOOR).  The synthetic output gradients are N(0, 1), so a row's
# gradient element is an fp32 sum of O(1) terms with an absolute error near 1e-7 whatever the sum comes to.
# When a few terms cancel (g = 1e-3 from three terms of size 1, seen with max pooling on a table of dim 4,
# where a single element carries the whole row gradient) m = mean(g^2) is tiny and that absolute error is
# 1e-4 of it; the floor keeps the bar at 1e-8 absolute there, far below any lost or misplaced contribution
# (at least 1/D of a squared gradient, ~2e-3).
M_FLOOR = 1e-3


class Tally:
    """vectors (rows, pooled slices) that missed the plain bar and were accepted on the peak scale"""

    def __init__(self):
        self.vectors = 0          # how many
        self.checked = 0          # out of how many compared
        self.worst_plain = 0.0    # largest error / plain bar seen on any vector (<= 1: within the stated tolerance)

    def as_dict(self):
        return {"vectors_on_peak_scale": self.vectors, "vectors_compared": self.checked,
                "worst_error_over_plain_bar": self.worst_plain}


def vec_err(got: np.ndarray, ref: np.ndarray, floor, peak=None) -> float:
    """largest norm-wise relative error over the rows of two [n, d] arrays; floor: a number or one per row;
    peak: per row, a magnitude the scale must not fall below (None: none)"""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    scale = np.maximum(np.abs(ref).max(axis=-1), floor)
    if peak is not None:
        scale = np.maximum(scale, peak)
    return float((np.abs(got - ref).max(axis=-1) / scale).max()) if got.size else 0.0


def check_vectors(got: np.ndarray, ref: np.ndarray, tol: float, floor, peak, tally: Tally, what: str):
    """Every row of got against ref on the plain bar  max_d|got - ref| <= tol * max(max_d|ref|, floor).
    peak (per row, or None): rows that miss the plain bar may pass on the scale max(.., peak) instead and
    are counted in `tally`; with peak None a miss is a failure."""
    if not got.size:
        return
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    err = np.abs(got - ref).max(axis=-1)
    scale = np.maximum(np.abs(ref).max(axis=-1), floor)
    ratio = err / (tol * scale)
    if tally is not None:
        tally.checked += int(ratio.size)
        tally.worst_plain = max(tally.worst_plain, float(ratio.max()))
    bad = ratio > 1.0
    if not bad.any():
        return
    assert peak is not None, f"{what} off by {float((err / scale).max()):.3e} (bar {tol:g})"
    wide = np.maximum(scale[bad], np.asarray(peak, dtype=np.float64)[bad] if np.ndim(peak) else peak)
    e = float((err[bad] / wide).max())
    assert e <= tol, f"{what} off by {e:.3e} even on the peak scale (bar {tol:g}); {float((err / scale).max()):.3e} on the plain one"
    if tally is not None:
        tally.vectors += int(bad.sum())


def make_backing(cfg, device="cpu"):
    """Initial tables for both sides: numpy copies for the oracle, pinned tensors for the GPU."""
    Wn, Mn, Wp, Mp = [], [], [], []
    for t, tc in enumerate(cfg.tables):
        dt = torch.float32 if tc.dtype == synth.FP32 else torch.float16
        wp = torch.empty(tc.rows, tc.dim, dtype=dt, pin_memory=True)
        synth.init_table(cfg, t, device=device, out=wp)
        mp = torch.zeros(tc.rows, dtype=torch.float32, pin_memory=True)
        Wp.append(wp)
        Mp.append(mp)
        Wn.append(wp.numpy().copy())
        Mn.append(mp.numpy().copy())
    return Wn, Mn, Wp, Mp


def _canon(arrs):
    """event arrays -> rows sorted lexicographically (events are compared as sets)"""
    m = np.stack([np.asarray(a, dtype=np.int64) for a in arrs], axis=1) if len(arrs[0]) else np.zeros((0, len(arrs)), np.int64)
    return m[np.lexsort(m.T[::-1])] if m.shape[0] else m


def gpu_snapshot(g, T: int):
    """counters, event sets and cache state of the library right after a prefetch"""
    return {"stats": g.stats()["last"],
            "events": {k: _canon(g.events(k)) for k in ("hit", "insert", "bypass")},
            "state": [g.cache_state(t) for t in range(T)],
            "freq": [g.cache_freq(t) for t in range(T)],
            "l2": [g.second_level_state(t) for t in range(T)], "l2_stats": g.second_level_stats()[0]}


def compare_cache_step(o: Oracle, snap, T: int, ctx: str):
    so, sg = o.stats()[0], snap["stats"]
    assert so == sg, f"{ctx}: counters differ: oracle {so} gpu {sg}"
    for kind in ("hit", "insert", "bypass"):
        eo, eg = _canon(o.events(kind)), snap["events"][kind]
        assert eo.shape == eg.shape and np.array_equal(eo, eg), f"{ctx}: {kind} events differ ({len(eo)} vs {len(eg)})"
    for t in range(T):
        to, tso = o.cache_state(t)
        tg, tsg = snap["state"][t]
        assert np.array_equal(to, tg), f"{ctx}: tags of table {t} differ"
        assert np.array_equal(tso, tsg), f"{ctx}: timestamps of table {t} differ"
        assert np.array_equal(o.cache_freq(t), snap["freq"][t]), f"{ctx}: lookup counts of table {t} differ"
        t2o, ts2o = o.second_level_state(t)
        t2g, ts2g = snap["l2"][t]
        assert np.array_equal(t2o, t2g), f"{ctx}: second-level tags of table {t} differ"
        assert np.array_equal(ts2o, ts2g), f"{ctx}: second-level timestamps of table {t} differ"
    assert o.second_level_stats()[0] == snap["l2_stats"], f"{ctx}: second-level counters differ: oracle {o.second_level_stats()[0]} gpu {snap['l2_stats']}"


def bag_peaks(cfg, o: Oracle, idx: np.ndarray, off: np.ndarray):
    """per table, per bag: the largest peak (see the header) among the rows the bag looks up; 0 for an empty bag"""
    B, res = (len(off) - 1) // cfg.num_tables, []
    for t in range(cfg.num_tables):
        o_t = off[t * B:(t + 1) * B + 1]
        pk = o.row_peak(t)[idx[o_t[0]:o_t[-1]]]
        out = np.zeros(B, dtype=np.float32)
        full = np.flatnonzero(np.diff(o_t) > 0)
        if len(full):
            out[full] = np.maximum.reduceat(pk, (o_t[full] - o_t[0]))
        res.append(out)
    return res


def compare_forward(cfg, out_o: np.ndarray, out_g: np.ndarray, ctx: str, peaks=None, tally: Tally = None):
    """peaks (fp16 storage under max pooling, where one row's element is the pooled element): bag_peaks()"""
    col = 0
    for t, tc in enumerate(cfg.tables):
        check_vectors(out_g[:, col:col + tc.dim], out_o[:, col:col + tc.dim], TOL[tc.dtype], 1e-3 * cfg.init_std,
                      peaks[t] if peaks is not None and tc.dtype == synth.FP16 else None, tally,
                      f"{ctx}: pooled output of table {t}")
        col += tc.dim


def compare_argmax(cfg, o: Oracle, idx: np.ndarray, off: np.ndarray, arg_g: np.ndarray, out_g: np.ndarray, ctx: str):
    """Between the oracle's forward and its update.  Returns the number of pooled elements whose maximum
    the library took from another row than the oracle, each verified to be a near-tie: the oracle's values of
    the two rows differ by no more than the bar allows the stored values to differ.  The library's pooled
    value must be that of the row it chose.  out_g is patched at those elements (they were checked here)."""
    a_o = o.argmax()
    assert a_o.shape == arg_g.shape
    B = (len(off) - 1) // cfg.num_tables
    cols = np.cumsum([0] + [tc.dim for tc in cfg.tables])
    flips = np.argwhere(a_o != arg_g)
    rows_seen = {}
    peak = [o.row_peak(t) for t in range(cfg.num_tables)] if len(flips) else None
    for b, c in flips:
        t = int(np.searchsorted(cols, c, side="right") - 1)
        tc, d = cfg.tables[t], int(c - cols[t])
        lo, hi = int(off[t * B + b]), int(off[t * B + b + 1])
        assert 0 <= arg_g[b, c] < hi - lo and a_o[b, c] >= 0, f"{ctx}: bag {b} of table {t}: position {arg_g[b, c]} is not in the bag"
        r_o, r_g = int(idx[lo + a_o[b, c]]), int(idx[lo + arg_g[b, c]])
        assert r_o != r_g, f"{ctx}: bag {b} of table {t}, element {d}: row {r_o} is looked up twice and the later lookup was taken"
        for r in (r_o, r_g):
            if (t, r) not in rows_seen:
                rows_seen[(t, r)] = o.read_row(t, r)[0]
        w_o, w_g = rows_seen[(t, r_o)], rows_seen[(t, r_g)]
        floor = 1e-3 * cfg.init_std
        s_o, s_g = max(np.abs(w_o).max(), peak[t][r_o], floor), max(np.abs(w_g).max(), peak[t][r_g], floor)
        band = TOL[tc.dtype] * (s_o + s_g)
        assert 0.0 <= w_o[d] - w_g[d] <= band, \
            f"{ctx}: bag {b} of table {t}, element {d}: took row {r_g} ({w_g[d]!r}) where row {r_o} ({w_o[d]!r}) is larger by more than the bar"
        assert abs(float(out_g[b, c]) - w_g[d]) <= TOL[tc.dtype] * s_g, \
            f"{ctx}: bag {b} of table {t}, element {d}: pooled value {float(out_g[b, c])!r} is not that of the row that supplied it (row {r_g}: {w_g[d]!r})"
        out_g[b, c] = w_o[d]
    return len(flips)


def first_bags(idx: torch.Tensor, off: torch.Tensor, T: int, n: int):
    """the batch made of the first n bags of every table of a table-major CSR batch"""
    B = (off.numel() - 1) // T
    parts, lens = [], []
    for t in range(T):
        lo, hi = int(off[t * B]), int(off[t * B + n])
        parts.append(idx[lo:hi])
        lens.append(off[t * B + 1:t * B + n + 1] - off[t * B:t * B + n])
    new_off = torch.cat([torch.zeros(1, dtype=torch.int64), torch.cumsum(torch.cat(lens), 0)])
    return torch.cat(parts).contiguous(), new_off.contiguous()


def compare_backing(cfg, Wn, Mn, Wp, Mp, ctx: str, only=None, peak=None, tally: Tally = None):
    """only[t]: boolean mask of the rows to compare (deferred initialisation: the rows that have a value;
    the others must still hold the NaN they were filled with, on both sides).  peak[t] (or None): per row,
    the wider scale that fp16 rows may fall back on (see the header); never used for fp32 storage."""
    step = 1 << 21  # rows per comparison chunk (keeps the fp64 temporaries small)
    for t, tc in enumerate(cfg.tables):
        wg, mg = Wp[t].numpy(), Mp[t].numpy()
        if only is not None:
            keep = only[t].astype(bool)
            assert np.isnan(wg[~keep].astype(np.float32)).all() and np.isnan(Wn[t][~keep].astype(np.float32)).all(), \
                f"{ctx}: a row of table {t} that was never read has been written"
            check_vectors(wg[keep], Wn[t][keep], TOL[tc.dtype], 1e-3 * cfg.init_std,
                          peak[t][keep] if peak is not None and tc.dtype == synth.FP16 else None, tally,
                          f"{ctx}: initialised rows of table {t}")
            em = vec_err(mg[:, None], Mn[t][:, None], floor=M_FLOOR)
            assert em <= 1e-5, f"{ctx}: accumulators of table {t} off by {em:.3e}"
            continue
        for r0 in range(0, tc.rows, step):
            r1 = min(tc.rows, r0 + step)
            check_vectors(wg[r0:r1], Wn[t][r0:r1], TOL[tc.dtype], 1e-3 * cfg.init_std,
                          peak[t][r0:r1] if peak is not None and tc.dtype == synth.FP16 else None, tally,
                          f"{ctx}: rows {r0}..{r1} of table {t}")
            em = vec_err(mg[r0:r1, None], Mn[t][r0:r1, None], floor=M_FLOOR)
            assert em <= 1e-5, f"{ctx}: accumulators {r0}..{r1} of table {t} off by {em:.3e}"


def compare_backing_touched(cfg, Wn, Mn, Wp, Mp, touched, ctx: str, tally: Tally = None):
    """For tables too large to widen row by row: the rows some batch looked up (touched[t]: sorted row ids) are
    held against the bar like everywhere else; all other rows must be bit for bit what both sides started from
    (checked by one whole-table byte comparison after the touched rows have been made equal); accumulators of
    all rows against theirs."""
    for t, tc in enumerate(cfg.tables):
        wg, mg = Wp[t].numpy(), Mp[t].numpy()
        rows = touched[t]
        check_vectors(wg[rows], Wn[t][rows], TOL[tc.dtype], 1e-3 * cfg.init_std, None, tally, f"{ctx}: touched rows of table {t}")
        Wn[t][rows] = wg[rows]
        assert torch.equal(torch.from_numpy(wg.view(np.int16 if tc.dtype == synth.FP16 else np.int32)),
                           torch.from_numpy(Wn[t].view(np.int16 if tc.dtype == synth.FP16 else np.int32))), \
            f"{ctx}: a row of table {t} that no batch looked up has changed"
        step = 1 << 24
        for r0 in range(0, tc.rows, step):
            em = vec_err(mg[r0:r0 + step, None], Mn[t][r0:r0 + step, None], floor=M_FLOOR)
            assert em <= 1e-5, f"{ctx}: accumulators {r0}.. of table {t} off by {em:.3e}"


def run_parity(cfg, steps: int, order: str = "serial", overlap: bool = True, check_every: int = 1, device="cuda",
               oracle_threads: int = 8, max_lookups: int = None, init_device="cpu", policy: str = "lru",
               pooling: str = "sum", second_level_factor: int = 0, max_batch: int = None, deferred_init=None,
               flush_every: int = 0, misuse: int = 0, vary_batch: int = 0, touched_only: bool = False,
               backing_throttle_ns: int = 0, probe_min_windows: int = 0):
    """order: 'serial'   prefetch(k) forward(k) backward(k)
              'inline'   forward(k) (prefetches itself) backward(k)
              'ahead'    prefetch(k+1) is issued between forward(k) and backward(k)
              'early'    prefetch(k+1) is issued before forward(k)
              'pipeD'    pipeline D batches deep (tbe_set_prefetch_depth): the batches up to k+D are prefetched before
                         forward(k); the oracle locks the ways of the D batches before the current one as well
    misuse = seed (0: off): between the regular calls, calls that the library must refuse -- an update with
    nothing forwarded, a second forward, a flush with a batch in flight, a forward whose buffers are not those
    of the pending prefetch, a batch above the sizes given at creation, a change of policy or pooling after
    the first batch -- each checked for its error code; the run must come out as if they had not been made.
    vary_batch = seed (0: off): every step trains on the first n bags of each table only, n drawn per step from
    1..batch (the library is created for the full batch).
    flush_every = n ('serial' and 'inline' only, where no batch is in flight between steps): both sides
    flush after every n-th step, the backing tiers are compared, and training goes on.
    backing_throttle_ns: the library's emulation of a slower backing tier (timing only: nothing may change).
    probe_min_windows: tbe_set_probe_grouping (tuning only: nothing may change); 1 makes the probe group the sets of
    small models, which it otherwise takes a wavefront each.
    Cache state, counters and event sets are compared after every `check_every`-th
    prefetch (the library's snapshot is taken right after its prefetch call, the oracle,
    which is strictly sequential, is compared when it reaches that batch)."""
    from paper_2305_01515_amd.tbe import TBE

    T = cfg.num_tables
    Wn, Mn, Wp, Mp = make_backing(cfg, device=init_device)
    if deferred_init is not None:  # (seed, std): the tables start without values; nothing may read the NaN
        for w, wn in zip(Wp, Wn):
            w.fill_(float("nan"))
            wn.fill(np.nan)
    slots = [tc.cache_slots for tc in cfg.tables]
    slots2 = [second_level_factor * (s // cfg.ways) * cfg.ways for s in slots] if second_level_factor else None
    pipe_depth = int(order[4:]) if order.startswith("pipe") else 0
    o = Oracle(Wn, Mn, slots, cfg.ways, threads=oracle_threads, policy=policy, pooling=pooling, second_level_slots=slots2,
               deferred_init=deferred_init, prefetch_lock=pipe_depth if pipe_depth >= 2 else 0)
    stream = synth.BatchStream(cfg, device="cpu")
    batches = [stream.next() for _ in range(steps)]
    sizes = [cfg.batch] * steps
    if vary_batch:
        vr = np.random.default_rng(vary_batch)
        sizes = [int(vr.choice([1, cfg.batch, int(vr.integers(1, cfg.batch + 1))])) for _ in range(steps)]
        batches = [first_bags(i, f, T, n) for (i, f), n in zip(batches, sizes)]
    if max_lookups is None:
        max_lookups = max(int(b[0].numel()) for b in batches) + 1
    g = TBE(Wp, Mp, slots, cfg.ways, max_batch or cfg.batch, max_lookups, overlap=overlap, policy=policy, pooling=pooling,
            second_level_factor=second_level_factor, deferred_init=deferred_init)
    if backing_throttle_ns:
        g.set_backing_throttle(backing_throttle_ns)
    if probe_min_windows:
        g.set_probe_grouping(probe_min_windows)
    if pipe_depth:
        g.set_prefetch_depth(pipe_depth)
    dev = [(i.to(device), f.to(device)) for i, f in batches]
    snaps = {}

    def gpu_prefetch(s, explicit=True):
        if explicit:
            g.prefetch(*dev[s])
        if s % check_every == 0 or s == steps - 1:
            snaps[s] = gpu_snapshot(g, T)

    parted = {"at": None, "elements": 0}
    tally = Tally()
    peak_allowed = pooling == "max"  # the wider scale is for fp16 rows under max pooling only (see the header)

    from paper_2305_01515_amd.tbe import TbeError, lib
    poke_rng = np.random.default_rng(misuse)
    poked = {"n": 0}
    EORDER, ELIMIT, EMISMATCH = -3, -5, -6

    def refused(code, fn, *args):
        try:
            fn(*args)
        except TbeError as e:
            assert e.code == code, f"refused with {e.code}, expected {code}: {e}"
            poked["n"] += 1
            return
        raise AssertionError(f"{getattr(fn, '__name__', fn)} was accepted where it must be refused")

    def set_mode(which, value):
        rc = getattr(lib(), which)(g._h, value)
        if rc:
            raise TbeError(rc, which)

    def poke(stage, idx=None, off=None):
        if not misuse or poke_rng.random() < 0.4:
            return
        zero_go = torch.zeros(cfg.batch, cfg.sum_dim, device=device)
        if stage == "not forwarded":
            choice = int(poke_rng.integers(0, 4))
            if choice == 0:
                refused(EORDER, g.backward_update, zero_go, cfg.lr, cfg.eps)
            elif choice == 1:
                refused(EORDER, g.argmax)
            elif choice == 2 and poked.get("started"):
                refused(EORDER, set_mode, "tbe_set_policy", 1)
            elif order in ("serial", "ahead", "early") and idx.numel():  # the batch's prefetch is pending: other buffers are a mismatch
                refused(EMISMATCH, g.forward, idx.clone(), off)
        else:  # a forwarded batch waits for its update
            choice = int(poke_rng.integers(0, 5))
            if choice == 0:
                refused(EORDER, g.forward, idx, off)
            elif choice == 1:
                refused(EORDER, g.flush)
            elif choice == 2:
                refused(EORDER, set_mode, "tbe_set_pooling", 1)
            elif choice == 3 and pooling != "max":
                refused(EORDER, g.argmax)
            elif choice == 4:
                too_many = torch.zeros(max_lookups + 1, dtype=torch.int64, device=device)
                refused(ELIMIT, g.prefetch, too_many, torch.zeros_like(off))

    def gpu_forward(idx, off):
        poke("not forwarded", idx, off)
        out = g.forward(idx, off)
        poked["started"] = True  # from the first batch on the modes are fixed
        arg = g.argmax() if pooling == "max" else None
        poke("forwarded", idx, off)
        return out, arg

    def oracle_step(s, res_g):
        out_g, arg_g = res_g
        idx, off = batches[s]
        o.prefetch(idx.numpy(), off.numpy())
        if s in snaps:
            compare_cache_step(o, snaps.pop(s), T, f"step {s + 1}")
        out_o = o.forward()
        if parted["at"] is None:
            out_g = out_g.cpu().numpy()
            if arg_g is not None:
                n = compare_argmax(cfg, o, idx.numpy(), off.numpy(), arg_g.cpu().numpy(), out_g, f"step {s + 1}")
                if n:
                    parted["at"], parted["elements"] = s + 1, n
            compare_forward(cfg, out_o, out_g, f"step {s + 1}",
                            peaks=bag_peaks(cfg, o, idx.numpy(), off.numpy()) if peak_allowed else None, tally=tally)
        o.backward_update(synth.grad_out(cfg, s + 1)[:sizes[s]].numpy(), cfg.lr, cfg.eps)

    pushed = 0
    for s in range(steps):
        go = synth.grad_out(cfg, s + 1)[:sizes[s]].to(device)
        idx, off = dev[s]
        if order == "serial":
            gpu_prefetch(s)
            out = gpu_forward(idx, off)
            g.backward_update(go, cfg.lr, cfg.eps)
        elif order == "inline":
            out = gpu_forward(idx, off)
            gpu_prefetch(s, explicit=False)
            g.backward_update(go, cfg.lr, cfg.eps)
        elif order == "ahead":
            if s == 0:
                gpu_prefetch(0)
            out = gpu_forward(idx, off)
            if s + 1 < steps:
                gpu_prefetch(s + 1)
            g.backward_update(go, cfg.lr, cfg.eps)
        elif order.startswith("pipe"):  # pipeN: a pipeline N batches deep (the oracle locks N batches as well)
            depth = int(order[4:])
            while pushed < min(steps, s + 1 + depth):
                gpu_prefetch(pushed)
                pushed += 1
            out = gpu_forward(idx, off)
            g.backward_update(go, cfg.lr, cfg.eps)
        elif order.startswith("deep"):  # deepN: a queue that accepts N batches ahead of training
            depth = int(order[4:])
            if s == 0:
                g.set_prefetch_queue(depth)
            while pushed < min(steps, s + 1 + depth):
                g.prefetch(*dev[pushed])
                pushed += 1
            out = gpu_forward(idx, off)
            g.backward_update(go, cfg.lr, cfg.eps)
        elif order == "early":
            if s == 0:
                gpu_prefetch(0)
            if s + 1 < steps:
                gpu_prefetch(s + 1)
            out = gpu_forward(idx, off)
            g.backward_update(go, cfg.lr, cfg.eps)
        else:
            raise ValueError(order)
        oracle_step(s, out)
        if flush_every and (s + 1) % flush_every == 0 and s + 1 < steps:
            assert order in ("serial", "inline")
            o.flush()
            g.flush()
            if parted["at"] is None:
                only = [o.initialised(t) for t in range(T)] if deferred_init is not None else None
                compare_backing(cfg, Wn, Mn, Wp, Mp, f"flush after step {s + 1}", only=only,
                                peak=[o.row_peak(t) for t in range(T)] if peak_allowed else None, tally=tally)
    assert not snaps
    # final cache state must agree whatever the call order was
    for t in range(T):
        to, tso = o.cache_state(t)
        tg, tsg = g.cache_state(t)
        assert np.array_equal(to, tg) and np.array_equal(tso, tsg), f"final cache state of table {t} differs"
        assert np.array_equal(o.cache_freq(t), g.cache_freq(t)), f"final lookup counts of table {t} differ"
        for a, b in zip(o.second_level_state(t), g.second_level_state(t)):
            assert np.array_equal(a, b), f"final second-level state of table {t} differs"
    assert o.second_level_stats()[1] == g.second_level_stats()[1], "total second-level counters differ"
    so, sg = o.stats()[1], g.stats()["total"]
    assert so == sg, f"total counters differ: oracle {so} gpu {sg}"
    o.flush()
    g.flush()
    only = None
    if deferred_init is not None:
        only = [o.initialised(t) for t in range(T)]
        for t in range(T):
            assert np.array_equal(only[t], g.initialised(t)), f"rows of table {t} that have a value differ"
    if parted["at"] is None and touched_only:
        # touched_only: tables of tens of GiB; rows that were looked up against the bar, the rest bit for bit
        assert deferred_init is None and not peak_allowed
        touched = [np.unique(np.concatenate([i.numpy()[int(f[t * (len(f) - 1) // T]):int(f[(t + 1) * (len(f) - 1) // T])]
                                             for i, f in batches])) for t in range(T)]
        compare_backing_touched(cfg, Wn, Mn, Wp, Mp, touched, "after flush", tally=tally)
    elif parted["at"] is None:
        compare_backing(cfg, Wn, Mn, Wp, Mp, "after flush", only=only,
                        peak=[o.row_peak(t) for t in range(T)] if peak_allowed else None, tally=tally)
    if not peak_allowed or all(tc.dtype == synth.FP32 for tc in cfg.tables):
        assert tally.vectors == 0
    st = g.stats()
    st["tolerance"] = tally.as_dict()
    st["parted_at"], st["parted_elements"] = parted["at"], parted["elements"]
    st["refused_calls"] = poked["n"]
    st["second_level_total"] = g.second_level_stats()[1]
    st["prefetch_depth"], st["rows_from_copies"] = g.prefetch_depth()
    g.close()
    o.close()
    return st
