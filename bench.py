#!/usr/bin/env python3
"""Benchmark of the cached embedding-bag training path on one MI355X.

A "step" is one pass of the whole hot path over one batch: prefetch (dedup, probe/LRU,
compaction, write-back + fill), pooled forward, backward with fused row-wise Adagrad.
The workload is the 32-table configuration (32 x 1M rows x dim 128 fp16, batch 8192,
pooling Poisson(30), Zipf 1.1, 64-way cache holding 5 % of the rows, backing tier in
pinned host memory, next-batch prefetch issued ahead of training).  All inputs of the
timed steps are generated beforehand and resident in HBM.

Prints ONE JSON line; the comments beside the fields below say what each one is.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
HOST_LINK_PEAK_GBS = 64.0  # PCIe Gen5 x16, per direction


def algorithmic_bytes(cfg, lookups_per_table, uniques, batch):
    """Bytes the method itself must move per step: rows once per lookup, location words and pooled output in the
    forward; rows read and written once per distinct row, accumulators and the output gradient once in the backward.
    Returns (forward, backward, gradient rows if counted per lookup, forward with every distinct row counted once)."""
    from paper_2305_01515_amd import synth
    from paper_2305_01515_amd.accounting import eq3_bytes_per_lookup
    T = len(cfg.tables)
    # Eq. 3 counts a row twice per lookup (forward and backward): the forward's half of it
    rows_fwd = sum(lookups_per_table[t] * eq3_bytes_per_lookup(cfg.tables[t].dim, 4 if cfg.tables[t].dtype == synth.FP32 else 2) // 2
                   for t in range(T))
    rb_mean = sum(tc.dim * (4 if tc.dtype == synth.FP32 else 2) for tc in cfg.tables) / T
    grad_per_lookup = sum(lookups_per_table[t] * cfg.tables[t].dim * 4 for t in range(T))
    io = 4 * batch * cfg.sum_dim                                   # pooled output / grad_out, once
    fwd = rows_fwd + 4 * sum(lookups_per_table) + io               # rows per lookup (Eq. 3) + locations + output
    bwd = uniques * (2 * rb_mean + 8) + io                         # row read-modify-write + accumulator + grad_out once
    fwd_unique = uniques * rb_mean + 4 * sum(lookups_per_table) + io  # what HBM has to deliver when repeats hit the caches
    return fwd, bwd, grad_per_lookup, fwd_unique


def sources_sha():
    """sha-256 (16 hex digits) over the HIP sources the library is built from: names a build"""
    import hashlib
    d = os.path.join(ROOT, "paper_2305_01515_amd", "csrc")
    h = hashlib.sha256()
    for n in sorted(os.listdir(d)):
        if n.endswith((".hip", ".h")):
            h.update(n.encode())
            h.update(open(os.path.join(d, n), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel_substr):
    """HBM bytes per launch of a kernel from the committed rocprofv3 --pmc summary
    (profiles/bench_main_pmc.txt: FETCH_SIZE / WRITE_SIZE scaled by the copy-kernel factors) -- only when that
    summary was taken with the sources this run is built from (its `sources_sha` line), else None: counter
    figures of another build beside this run's timings would say nothing."""
    path = os.path.join(ROOT, "profiles", "bench_main_pmc.txt")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    sha = [l.split()[1] for l in lines if l.startswith("sources_sha ") and len(l.split()) > 1]
    if not sha or sha[0] != sources_sha():
        return None
    tot = None
    for line in lines:
        f = line.split()
        if len(f) >= 4 and f[0] == "traffic" and f[1] == kernel_substr:
            tot = (tot or 0.0) + float(f[2]) + float(f[3])
    return tot


def measured_peaks(torch):
    """What this machine delivers with plain copies (context for the two rooflines): a 1 GiB
    device-to-device copy (read + write bytes) and 1 GiB pinned host copies each way."""
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    h = torch.empty(n, dtype=torch.uint8, pin_memory=True)

    def rate(fn, nbytes, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9

    out = {"hbm_copy_GBps": rate(lambda: b.copy_(a), 2 * n),
           "h2d_GBps": rate(lambda: a.copy_(h, non_blocking=True), n),
           "d2h_GBps": rate(lambda: h.copy_(a, non_blocking=True), n)}
    del a, b, h
    return out


def cpu_baseline(cfg, W0, batches, grads, threads):
    """The oracle as it stands, timed on this machine's host cores on the first batches."""
    import numpy as np
    from oracle import Oracle
    Wn = [w.numpy().copy() for w in W0]
    Mn = [np.zeros(w.shape[0], dtype=np.float32) for w in W0]
    o = Oracle(Wn, Mn, [t.cache_slots for t in cfg.tables], cfg.ways, threads=threads)
    n = 0
    t0 = time.perf_counter()
    for (idx, off), g in zip(batches, grads):
        o.prefetch(idx, off)
        o.forward()
        o.backward_update(g, cfg.lr, cfg.eps)
        n += idx.size
        if time.perf_counter() - t0 > 20.0:
            break
    dt = time.perf_counter() - t0
    o.close()
    return n / dt, n


def all_hit_control(TBE, cfg, Wp, Mp, batch, grads, out, max_n, hit_bytes, overlap, inputs_ready=True, steps=10):
    """The same shapes with no miss traffic at all: a cache as large as the tables and one batch
    replayed, so every distinct row hits.  Prefetch stage, forward and backward run pipelined as in the
    timed region; the host link is idle.  Not part of `value`."""
    import torch
    g = TBE(Wp, Mp, [tc.rows + cfg.ways for tc in cfg.tables], cfg.ways, cfg.batch, max_n + 1, overlap=overlap)
    g.set_inputs_ready(inputs_ready)

    def run(n):
        for s in range(n):
            g.prefetch(*batch)
            g.forward(batch[0], batch[1], out)
            g.backward_update(grads[s % len(grads)], cfg.lr, cfg.eps)

    g.prefetch(*batch)
    run(3)  # the first step inserts the rows, the next ones hit
    torch.cuda.synchronize()
    s0 = g.stats()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    s1 = g.stats()
    g.forward(batch[0], batch[1], out)
    g.backward_update(grads[0], cfg.lr, cfg.eps)
    torch.cuda.synchronize()
    g.close()
    n = int(batch[0].numel())
    uniq = s1["total"]["uniques"] - s0["total"]["uniques"]
    return {"what": "cache >= tables and one batch replayed: every row hits, host link idle; prefetch stage + forward + "
                    "backward pipelined", "steps": steps, "ms_per_step": dt * 1e3, "lookups_per_s": n / dt,
            "hit_rate_unique": (s1["total"]["hits"] - s0["total"]["hits"]) / max(1, uniq),
            "link_bytes_per_step": (s1["h2d_bytes"] - s0["h2d_bytes"] + s1["d2h_bytes"] - s0["d2h_bytes"]) / steps,
            "hit_path_bytes": hit_bytes, "frac": hit_bytes / dt / 1e9 / HBM_PEAK_GBS}


def locality_sweep(args):
    """The (index distribution, cache size) sweep of the locality configuration: 1 table x 100M rows x
    dim 64 fp16, batch 32768, pooling 32; for every point 100 warm-up steps, then `--steps` measured
    steps, pipelined.  One table in pinned memory serves all points (the values do not matter to the
    hit rates).  Prints one JSON line with the whole table."""
    import torch
    from paper_2305_01515_amd import synth
    from paper_2305_01515_amd.tbe import TBE
    dev = "cuda"
    warm, K = 100, args.steps
    base = synth.config_locality(None, 0.01)
    tc = base.tables[0]
    w = torch.empty(tc.rows, tc.dim, dtype=torch.float16, pin_memory=True)
    synth.init_table(base, 0, device=dev, out=w)
    m = torch.zeros(tc.rows, dtype=torch.float32, pin_memory=True)
    out = torch.empty(base.batch, base.sum_dim, dtype=torch.float32, device=dev)
    grads = [synth.grad_out(base, s + 1, device=dev) for s in range(4)]
    points = []
    for alpha in (None, 0.8, 1.0, 1.2, 1.4):
        stream = synth.BatchStream(synth.config_locality(alpha, 0.01), device=dev)
        batches = [stream.next() for _ in range(warm + K + 1)]
        max_n = max(int(b[0].numel()) for b in batches)
        for frac in (0.01, 0.02, 0.05, 0.10, 0.25):
            cfg = synth.config_locality(alpha, frac)
            g = TBE([w], [m], [cfg.tables[0].cache_slots], cfg.ways, cfg.batch, max_n + 1, overlap=not args.no_overlap,
                    policy=args.policy)
            g.set_inputs_ready(True)

            def run(lo, hi):
                for s in range(lo, hi):
                    g.prefetch(*batches[s + 1])
                    g.forward(batches[s][0], batches[s][1], out)
                    g.backward_update(grads[s % len(grads)], cfg.lr, cfg.eps)

            g.prefetch(*batches[0])
            run(0, warm)
            torch.cuda.synchronize()
            s0 = g.stats()
            t0 = time.perf_counter()
            run(warm, warm + K)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            s1 = g.stats()
            g.forward(batches[warm + K][0], batches[warm + K][1], out)
            g.backward_update(grads[0], cfg.lr, cfg.eps)
            torch.cuda.synchronize()
            g.close()
            tot = {k: s1["total"][k] - s0["total"][k] for k in s1["total"]}
            n = sum(int(batches[s][0].numel()) for s in range(warm, warm + K))
            points.append({"alpha": alpha, "cache_frac": frac, "hit_rate_unique": tot["hits"] / max(1, tot["uniques"]),
                           "hit_rate_lookup": tot["hit_lookups"] / max(1, tot["lookups"]),
                           "uniques_per_step": tot["uniques"] / K, "ms_per_step": dt / K * 1e3, "lookups_per_s": n / dt,
                           "h2d_GBps": (s1["h2d_bytes"] - s0["h2d_bytes"]) / dt / 1e9,
                           "d2h_GBps": (s1["d2h_bytes"] - s0["d2h_bytes"]) / dt / 1e9})
            print("point", points[-1], file=sys.stderr, flush=True)
    print(json.dumps({"metric": "locality sweep: hit rate and pooled lookups/s per (index distribution, cache size)",
                      "unit": "lookups/s", "n_gpus": 1, "steps": K, "warmup": warm, "data": "synthetic",
                      "dtype": "f16 storage / f32 accumulate",
                      "config": {"workload": "1 table x 100M rows x dim 64 fp16, batch 32768, pooling 32, 64-way cache, "
                                             "uniform / Zipf 0.8 / 1.0 / 1.2 / 1.4 x cache 1 / 2 / 5 / 10 / 25 % of rows",
                                 "policy": args.policy},
                      "sweep": points}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: 200 for the benchmark workload, as its configuration says; 20 for the others)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 10 / 5)")
    ap.add_argument("--tables", type=int, default=32, help="(debug) fewer tables than the named workload")
    ap.add_argument("--workload", default="main", choices=["main", "tiny", "capacity", "locality", "hetero", "locality_sweep"],
                    help="main = the benchmark workload; the others are the parity configurations, for reference "
                         "measurements only (no CPU baseline)")
    ap.add_argument("--alpha", type=float, default=1.0, help="locality: Zipf exponent, 0 = uniform")
    ap.add_argument("--cache-frac", type=float, default=0.05, help="locality: cached fraction of the rows")
    ap.add_argument("--policy", default="lru", choices=["lru", "lfu"],
                    help="replacement policy; lru is the benchmark's, lfu for the comparison the paper makes")
    ap.add_argument("--prefetch-depth", type=int, default=1,
                    help="pipeline this many batches deep (tbe_set_prefetch_depth; 1 = the benchmark's)")
    ap.add_argument("--backing-throttle-ns", type=int, default=0,
                    help="emulate a slower backing tier: the host-link kernel pauses this long per backing-tier row (0 = off)")
    ap.add_argument("--second-level", type=int, default=0,
                    help="factor of a second-level cache in pinned host memory (0 = none, the benchmark's)")
    ap.add_argument("--deferred-init", action="store_true",
                    help="rows get their initial values on first read, on the GPU (not the benchmark's setting)")
    ap.add_argument("--pooling", default="sum", choices=["sum", "mean", "max"], help="sum is the benchmark's")
    ap.add_argument("--resident-fraction", type=float, default=-1.0,
                    help="hetero: share of the HBM budget given to whole tables chosen by the placement solver "
                         "(Eq. 6); negative = plain split in proportion to lookups x dim")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--wait-for-compute", action="store_true",
                    help="leave the default ordering of tbe_prefetch behind the compute stream in place")
    ap.add_argument("--no-control", action="store_true", help="skip the all-hit control run after the benchmark "
                    "(so that a profile of the process holds the benchmark's launches only)")
    ap.add_argument("--no-overlap", action="store_true", help="run everything on one stream")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 200 if args.workload == "main" else 100 if args.workload == "locality_sweep" else 20
    if args.warmup is None:
        args.warmup = 10 if args.workload == "main" else 5
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2305_01515_amd import synth
    from paper_2305_01515_amd.tbe import TBE

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "locality_sweep":
        return locality_sweep(args)
    dev = "cuda"
    K, Wm = args.steps, args.warmup
    if args.workload == "main":
        cfg = synth.config_main(tables=args.tables)
        desc = ("32 tables x 1M rows x dim 128 fp16, batch 8192, pooling Poisson(30) in [1,200], Zipf 1.1, 64-way LRU "
                "cache 5% of rows in HBM, backing tier in pinned host memory, next-batch prefetch ahead of training")
    elif args.workload == "tiny":
        cfg = synth.config_tiny()
        desc = "4 tables x 100k rows x dim 64 fp32, batch 512, pooling 20, Zipf 1.05, 32-way cache 10% of rows"
    elif args.workload == "capacity":
        # the test box refuses to pin more than about 64 GiB of host memory, so half the rows
        # (and half the cache: the same 6.25 % of the rows); per-step shape unchanged
        cfg = synth.config_capacity(rows=1 << 25, cache_bytes=4 << 30)
        desc = ("8 tables x 32M rows x dim 128 fp16 (64 GiB in pinned host memory; half of the capacity-bound "
                "configuration's rows), 4 GiB 64-way cache, batch 65536, pooling Poisson(40), Zipf 1.05, 30% of each "
                "batch re-drawn from the previous 4 batches")
    elif args.workload == "hetero":
        # 1/10 of the rows of the heterogeneous configuration (its 175 GB do not fit the pinned memory of
        # the box), cache budget scaled alike; per-step shape unchanged
        cfg = synth.config_hetero(max_rows=5e6, cache_bytes=(16 << 30) // 10)
        probe = synth.BatchStream(cfg)
        _, off = probe.next()
        lk = [int(off[(t + 1) * cfg.batch] - off[t * cfg.batch]) for t in range(cfg.num_tables)]
        if args.resident_fraction < 0:
            synth.split_cache_budget(cfg, lk, cfg.cache_bytes)
            how = "split in proportion to lookups x dim"
        else:
            res = synth.place_and_split_cache_budget(cfg, lk, cfg.cache_bytes, args.resident_fraction)
            how = (f"{args.resident_fraction:.0%} of it for {len(res)} whole tables chosen by the placement solver, "
                   "the rest split in proportion to lookups x dim")
        desc = (f"100 tables, rows log-uniform in [1e4, 5e6] (1/10 of the heterogeneous configuration), dims 64/128/256 "
                f"fp16, pooling means 1..100, Zipf 0.9..1.3, batch 16384, 64-way cache of 1.6 GiB, {how}")
    else:
        cfg = synth.config_locality(args.alpha if args.alpha > 0 else None, args.cache_frac)
        desc = (f"1 table x 100M rows x dim 64 fp16, batch 32768, pooling 32, "
                f"{'uniform' if args.alpha <= 0 else 'Zipf %g' % args.alpha}, 64-way cache {args.cache_frac:.0%} of rows")
    if args.policy != "lru":
        desc = desc.replace("LRU ", "").replace("-way cache", "-way LFU cache")
    if args.workload != "main" or args.policy != "lru" or args.pooling != "sum" or args.second_level or args.deferred_init or args.backing_throttle_ns:
        args.no_cpu_baseline = True
    T = cfg.num_tables

    # plain copies for context -- not where the tables need all the pinned memory the box allows (the buffers
    # of the measurement stay in torch's pinned-memory cache)
    peaks = measured_peaks(torch) if args.workload != "capacity" else None

    # backing tier: pinned host tables, initialised on the GPU and copied over
    Wp, Mp = [], []
    for t, tc in enumerate(cfg.tables):
        w = torch.empty(tc.rows, tc.dim, dtype=torch.float32 if tc.dtype == synth.FP32 else torch.float16,
                        pin_memory=True)
        synth.init_table(cfg, t, device=dev, out=w)
        Wp.append(w)
        Mp.append(torch.zeros(tc.rows, dtype=torch.float32, pin_memory=True))
    torch.cuda.synchronize()

    # inputs of all steps, resident in HBM before anything is timed
    stream = synth.BatchStream(cfg, device=dev)
    ISO = 4  # extra steps after the timed region, run stage by stage for isolated kernel times
    batches = [stream.next() for _ in range(K + Wm + 1 + 2 * ISO)]
    grads = [synth.grad_out(cfg, s + 1, device=dev) for s in range(min(K + Wm, 6))]
    max_n = max(int(b[0].numel()) for b in batches)
    out = torch.empty(cfg.batch, cfg.sum_dim, dtype=torch.float32, device=dev)

    cpu = None
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        nb = 3
        v, n = cpu_baseline(cfg, Wp, [(b[0].cpu().numpy(), b[1].cpu().numpy()) for b in batches[:nb]],
                            [g.cpu().numpy() for g in grads[:nb]], threads)
        model = ""
        try:
            with open("/proc/cpuinfo") as f:
                model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
        except OSError:
            pass
        cpu = {"value": v, "unit": "lookups/s", "cores": threads, "kind": "oracle", "cpu_model": model,
               "host_cpus": os.cpu_count(),
               "sample": f"first batches of the same stream from a cold cache ({n} lookups), oracle -O2, OpenMP over tables"}

    g = TBE(Wp, Mp, [tc.cache_slots for tc in cfg.tables], cfg.ways, cfg.batch, max_n + 1, overlap=not args.no_overlap,
            policy=args.policy, pooling=args.pooling, second_level_factor=args.second_level,
            deferred_init=(cfg.seed, cfg.init_std) if args.deferred_init else None)

    D = args.prefetch_depth
    pushed = [0]

    def run(lo, hi):
        # the next batch (the next D batches) are prefetched ahead of the current batch's training
        for s in range(lo, hi):
            while pushed[0] < min(s + 1 + D, hi + 1):
                g.prefetch(*batches[pushed[0]])
                pushed[0] += 1
            g.forward(batches[s][0], batches[s][1], out)
            g.backward_update(grads[s % len(grads)], cfg.lr, cfg.eps)

    if args.backing_throttle_ns:
        g.set_backing_throttle(args.backing_throttle_ns)
    if D > 1:
        g.set_prefetch_depth(D)
    g.set_inputs_ready(not args.wait_for_compute)  # all index tensors were generated and synchronised above
    g.set_profiling(True)  # stage brackets from the first launch on, so that the means over all
    g.prefetch(*batches[0])  # launches can be compared with a rocprofv3 --stats run of this command
    pushed[0] = 1
    run(0, Wm)
    torch.cuda.synchronize()
    s0 = g.stats()
    l2_0 = g.second_level_stats() if args.second_level else None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(Wm, Wm + K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    s1 = g.stats()
    l2_1 = g.second_level_stats() if args.second_level else None
    BWD = ("backward_single", "backward_short", "backward_heavy", "backward_combine")
    STAGES = ("prefetch", "fill", "commit", "forward", "backward") + BWD
    first = {k: (Wm if k in ("forward", "backward") + BWD else Wm + 1) for k in STAGES}
    times = {k: g.stage_times(k)[first[k]:first[k] + K] for k in STAGES}  # the brackets of the timed steps

    # isolated pass (not part of `value`): the same kernels with nothing else on the GPU
    g.forward(batches[Wm + K][0], batches[Wm + K][1], out)
    g.backward_update(grads[0], cfg.lr, cfg.eps)
    torch.cuda.synchronize()
    for s in range(Wm + K + 1, Wm + K + 1 + ISO):
        g.prefetch(*batches[s])
        torch.cuda.synchronize()
        g.forward(batches[s][0], batches[s][1], out)
        torch.cuda.synchronize()
        g.backward_update(grads[s % len(grads)], cfg.lr, cfg.eps)
        torch.cuda.synchronize()
    iso = {k: float(np.mean(g.stage_times(k)[-ISO:])) for k in STAGES}
    all_launches = {k: float(np.mean(g.stage_times(k))) for k in STAGES}
    # once more with the whole-stage brackets only: the brackets around the backward's single kernels lie inside
    # the one around the whole backward and lengthen it by their own events
    g.set_profiling(2)
    for s in range(Wm + K + 1 + ISO, Wm + K + 1 + 2 * ISO):
        g.prefetch(*batches[s])
        torch.cuda.synchronize()
        g.forward(batches[s][0], batches[s][1], out)
        torch.cuda.synchronize()
        g.backward_update(grads[s % len(grads)], cfg.lr, cfg.eps)
        torch.cuda.synchronize()
    iso_detail_backward = iso["backward"]
    iso["forward"] = float(np.mean(g.stage_times("forward")))
    iso["backward"] = float(np.mean(g.stage_times("backward")))

    # the timed region trained batches Wm..Wm+K-1; it prefetched batches Wm+1..Wm+K (one ahead)
    lookups = sum(int(batches[s][0].numel()) for s in range(Wm, Wm + K))
    tot = {k: s1["total"][k] - s0["total"][k] for k in s1["total"]}
    npf = K  # one prefetch per timed step
    h2d = (s1["h2d_bytes"] - s0["h2d_bytes"]) / npf
    d2h = (s1["d2h_bytes"] - s0["d2h_bytes"]) / npf

    # per-table counts for the algorithmic bytes (from the offsets; uniques from the library's counters)
    off = batches[Wm][1].cpu()
    per_table = [int(off[(t + 1) * cfg.batch] - off[t * cfg.batch]) for t in range(T)]
    scale = (lookups / K) / max(1, sum(per_table))
    per_table = [p * scale for p in per_table]
    uniq = tot["uniques"] / npf
    fwd_b, bwd_b, grad_pl, fwd_uniq_b = algorithmic_bytes(cfg, per_table, uniq, cfg.batch)

    ms = {k: float(np.mean(v)) if v.size else 0.0 for k, v in times.items()}

    def gbs(nbytes, t_ms):
        return nbytes / (t_ms * 1e-3) / 1e9 if t_ms else 0.0

    # the whole backward, one bracket from before its first kernel to after its last
    bwd_ms, bwd_iso = ms["backward"], iso["backward"]
    hit_ms, hit_iso = ms["forward"] + bwd_ms, iso["forward"] + bwd_iso
    hit_b = fwd_b + bwd_b
    # the committed counter summary is of the benchmark workload only
    main32 = (args.workload == "main" and T == 32 and args.policy == "lru" and args.pooling == "sum"
              and not args.second_level and not args.deferred_init)
    fwd_traffic = measured_traffic("forward_kernel") if main32 else None
    bwd_traffic = {k: (measured_traffic(k + "_kernel") if fwd_traffic else None) for k in BWD}
    hit_traffic = (fwd_traffic + sum(bwd_traffic.values())) if fwd_traffic and all(bwd_traffic.values()) else None
    fill_ms = ms["fill"]
    link_gbs = max(h2d, d2h) / (fill_ms * 1e-3) / 1e9 if fill_ms else 0.0
    res = {
        "metric": "pooled lookups/s (fwd+bwd+update), achieved HBM GB/s, cache hit rate",
        "value": lookups / dt,
        "unit": "lookups/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": dt / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage / f32 accumulate" if cfg.tables[0].dtype == synth.FP16 else "f32", "data": "synthetic",
        "config": {"workload": desc,
                   "tables": T, "batch": cfg.batch, "lookups_per_step": lookups / K,
                   "overlap": not args.no_overlap, "policy": args.policy, "pooling": args.pooling,
                   "second_level_factor": args.second_level, "deferred_init": args.deferred_init,
                   "backing_throttle_ns": args.backing_throttle_ns, "prefetch_depth": D},
        # The dominant kernel of a step: transfer_kernel (write-back of parked victims beside the fetch-ahead of the
        # missed rows), bound by the host link.  achieved = bytes of the busier direction per launch / mean launch time,
        # measured live in the timed, pipelined region with HIP events on the link stream; peak = PCIe Gen5 x16 per
        # direction.  bytes_per_launch: the miss path's algorithmic bytes (inserted + bypassed rows in, evicted + bypassed
        # rows out, a row's bytes each), counted by the kernel itself.  traffic: HBM bytes of the kernel per launch from
        # the committed counter summary, null unless that summary is of this build.
        "roofline": {"kernel": "transfer_kernel (host link: write-back of parked victims + fetch-ahead of missed rows)",
                     "bound": "host_link", "achieved": link_gbs, "peak": HOST_LINK_PEAK_GBS, "unit": "GB/s",
                     "frac": link_gbs / HOST_LINK_PEAK_GBS, "traffic": measured_traffic("transfer_kernel") if main32 else None,
                     "bytes_per_launch": {"h2d": h2d, "d2h": d2h}, "ms_per_launch": fill_ms,
                     "h2d_GBps": gbs(h2d, fill_ms), "d2h_GBps": gbs(d2h, fill_ms),
                     "isolated": {"ms_per_launch": iso["fill"]}},
        # Forward kernel.  hbm: what HBM delivered -- counter traffic (committed summary of this build, else null) over
        # the launch time, against the 8 TB/s peak.  eq3_rate_GBps counts every row once per lookup (the paper's Eq. 3);
        # repeats of hot rows are served by L2, so it is a rate at L2 level and NOT a fraction of the HBM peak.
        "forward": {"kernel": "forward_kernel (pooled gather), %d lanes per row" % (cfg.tables[0].dim // (8 if cfg.tables[0].dtype == synth.FP16 else 4)),
                    "ms_per_launch": ms["forward"], "isolated_ms_per_launch": iso["forward"],
                    "eq3_bytes_per_launch": fwd_b, "eq3_rate_GBps": gbs(fwd_b, ms["forward"]),
                    "eq3_rate_isolated_GBps": gbs(fwd_b, iso["forward"]),
                    "unique_row_bytes_per_launch": fwd_uniq_b,
                    "hbm": {"traffic": fwd_traffic, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "achieved": gbs(fwd_traffic, ms["forward"]) if fwd_traffic else None,
                            "frac": gbs(fwd_traffic, ms["forward"]) / HBM_PEAK_GBS if fwd_traffic else None,
                            "isolated_frac": gbs(fwd_traffic, iso["forward"]) / HBM_PEAK_GBS if fwd_traffic else None}},
        # backward = single-lookup rows bag by bag / rows with 2..64 lookups / heavy rows through LDS tiles / their combine;
        # ms_total is the bracket around all of them, ms the brackets of the single kernels inside it (rocprofv3's
        # kernel durations are these, less the events' overhead)
        "backward": {"bound": "hbm", "bytes_per_step": bwd_b, "ms": {k: ms[k] for k in BWD}, "ms_total": bwd_ms,
                     "achieved": gbs(bwd_b, bwd_ms), "frac": gbs(bwd_b, bwd_ms) / HBM_PEAK_GBS,
                     "isolated": {"ms": {k: iso[k] for k in BWD}, "ms_total": bwd_iso,
                                  "ms_total_with_the_kernels_bracketed": iso_detail_backward, "achieved": gbs(bwd_b, bwd_iso),
                                  "frac": gbs(bwd_b, bwd_iso) / HBM_PEAK_GBS},
                     "traffic": bwd_traffic,
                     "traffic_over_compulsory": (sum(bwd_traffic.values()) / bwd_b) if bwd_traffic and all(bwd_traffic.values()) else None},
        # Hit path = forward + backward + update kernels of a step against the 8 TB/s HBM peak.  bytes: rows once per
        # lookup in the forward (Eq. 3), once per distinct row (read + write) in the backward.  frac_unique_rows counts
        # the forward's rows once per distinct row as well: the bytes HBM itself has to deliver.
        "hit_path": {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "ms_fwd_bwd": hit_ms, "bytes": hit_b, "lookups_per_s": (lookups / K) / (hit_ms * 1e-3) if hit_ms else 0.0,
                     "achieved": gbs(hit_b, hit_ms), "frac": gbs(hit_b, hit_ms) / HBM_PEAK_GBS,
                     "frac_unique_rows": gbs(fwd_uniq_b + bwd_b, hit_ms) / HBM_PEAK_GBS,
                     "isolated": {"ms_fwd_bwd": hit_iso, "lookups_per_s": (lookups / K) / (hit_iso * 1e-3) if hit_iso else 0.0,
                                  "achieved": gbs(hit_b, hit_iso), "frac": gbs(hit_b, hit_iso) / HBM_PEAK_GBS,
                                  "frac_unique_rows": gbs(fwd_uniq_b + bwd_b, hit_iso) / HBM_PEAK_GBS,
                                  # HBM bytes the counters saw for these kernels / their time: the bandwidth HBM delivered
                                  "traffic": hit_traffic,
                                  "traffic_frac": gbs(hit_traffic, hit_iso) / HBM_PEAK_GBS if hit_traffic else None}},
        "prefetch_stage_ms": ms["prefetch"], "commit_stage_ms": ms["commit"],
        "isolated_stage_ms": iso,
        # mean over every launch of the process (warm-up, timed, isolated): what rocprofv3 --stats averages
        "all_launches_stage_ms": all_launches,
        "cache": {"hit_rate_unique": tot["hits"] / max(1, tot["uniques"]),
                  "hit_rate_lookup": tot["hit_lookups"] / max(1, tot["lookups"]),
                  "bypass_frac_unique": tot["bypasses"] / max(1, tot["uniques"]),
                  "uniques_per_step": uniq, "inserts_per_step": tot["inserts"] / npf, "long_rows": s1["last_long_rows"],
                  "late_fetches_per_step": (s1["late_fetches"] - s0["late_fetches"]) / npf},
        "measured_peaks": peaks,  # plain copies on this machine, for context (the fractions above use the nominal peaks)
        "sources_sha": sources_sha(),
        # HBM the library holds beside the cache lines, in bytes: accumulators of all rows (4 B per row), the map of
        # rows whose backing-tier copy is momentarily stale (4 B per sort key), tags / timestamps / counts / slot
        # accumulators (16 B per slot) -- scales with the rows, not with the cache
        "hbm_footprint": {"cache_lines": sum(tc.cache_slots // cfg.ways * cfg.ways * tc.dim * (4 if tc.dtype == synth.FP32 else 2) for tc in cfg.tables),
                          "accumulators_all_rows": 4 * sum(tc.rows for tc in cfg.tables),
                          "stale_copy_map": 4 * sum(tc.rows for tc in cfg.tables),
                          "per_slot_state": 16 * sum(tc.cache_slots // cfg.ways * cfg.ways for tc in cfg.tables)},
        "cpu_baseline": cpu,
    }
    second_level = None
    if args.second_level:
        l2a, l2b = l2_0[1], l2_1[1]
        second_level = {k: (l2b[k] - l2a[k]) / npf for k in l2b}
        second_level["hit_rate_of_first_level_misses"] = (l2b["hits"] - l2a["hits"]) / max(1, tot["inserts"] + tot["bypasses"])
    g.close()
    if args.workload == "main" and not args.second_level and not args.no_control and not args.deferred_init and not args.backing_throttle_ns:
        res["all_hit_control"] = all_hit_control(TBE, cfg, Wp, Mp, batches[Wm + K], grads, out, max_n, hit_b,
                                                 not args.no_overlap, not args.wait_for_compute)
    if args.second_level:
        res["second_level"] = second_level
    print(json.dumps(res))


if __name__ == "__main__":
    main()
