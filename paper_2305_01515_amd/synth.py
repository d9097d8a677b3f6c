"""Seeded synthetic inputs shaped like the paper's workloads.

The paper measured on private production models and day-long access traces
(Section 4.1, Table 2); none of that is public.  What it states about them is
used here as the recipe: accesses follow a power law (Section 4.1, temporal
locality), rows are 64-256 elements wide (Section 4.2), a sample touches a few
tens of rows per table (Table 2, average pooling size), and table sizes spread
over orders of magnitude with the large tables being the cold ones (Fig. 1).

This module only *draws inputs*: table shapes, index/offset arrays, upstream
gradients and initial weights.  It contains none of the method's arithmetic
(no pooling, no optimizer, no cache logic) and is the only code that both the
CPU oracle's tests and the HIP path's tests call.  Everything is a pure
function of (config, seed, step); tensors are produced with torch so the same
recipe runs on the host or on a GPU (the two devices use different random
streams: an array is always generated once and handed to both sides).
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Tuple

import torch

FP32 = 0
FP16 = 1


@dataclasses.dataclass
class TableCfg:
    rows: int                 # H_t
    dim: int                  # D_t
    dtype: int                # FP32 / FP16 storage
    alpha: Optional[float]    # Zipf exponent; None = uniform
    pool_kind: str            # "fixed" | "poisson"
    pool_mean: float
    pool_lo: int = 0
    pool_hi: int = 200
    cache_slots: int = 0


@dataclasses.dataclass
class WorkloadCfg:
    name: str
    tables: List[TableCfg]
    batch: int
    ways: int
    steps: int
    seed: int
    reuse_frac: float = 0.0   # fraction of each batch re-drawn from recent batches
    reuse_window: int = 4
    lr: float = 0.01
    eps: float = 1e-8
    init_std: float = 0.01

    @property
    def sum_dim(self) -> int:
        return sum(t.dim for t in self.tables)

    @property
    def num_tables(self) -> int:
        return len(self.tables)


def _slots(rows: int, frac: float, ways: int) -> int:
    """Cache slots for a table: `frac` of its rows, rounded down to whole sets."""
    return (int(rows * frac) // ways) * ways


def config_tiny(seed: int = 0) -> WorkloadCfg:
    """4 tables x 100k rows x dim 64 fp32, batch 512, pooling 20, Zipf 1.05,
    32-way cache holding 10 % of the rows, 20 steps."""
    ways = 32
    tabs = [TableCfg(100_000, 64, FP32, 1.05, "fixed", 20, cache_slots=_slots(100_000, 0.10, ways))
            for _ in range(4)]
    return WorkloadCfg("tiny", tabs, batch=512, ways=ways, steps=20, seed=seed)


def config_main(seed: int = 1, tables: int = 32, rows: int = 1_000_000, batch: int = 8192,
                steps: int = 200) -> WorkloadCfg:
    """32 tables x 1M rows x dim 128 fp16, batch 8192, pooling Poisson(30) in
    [1, 200], Zipf 1.1, 64-way cache holding 5 % of the rows."""
    ways = 64
    tabs = [TableCfg(rows, 128, FP16, 1.1, "poisson", 30, 1, 200, cache_slots=_slots(rows, 0.05, ways))
            for _ in range(tables)]
    return WorkloadCfg("main", tabs, batch=batch, ways=ways, steps=steps, seed=seed)


def config_hetero(seed: int = 2, tables: int = 100, max_rows: float = 5e7, batch: int = 16384,
                  cache_bytes: int = 16 << 30, steps: int = 200) -> WorkloadCfg:
    """100 tables, rows log-uniform in [1e4, max_rows], dims from {64, 128, 256}
    fp16, pooling mean log-uniform in [1, 100], Zipf alpha uniform in
    [0.9, 1.3]; a cache budget split in proportion to lookups x dim.
    `split_cache_budget` assigns the slots once a sample batch is measured."""
    g = torch.Generator().manual_seed(seed * 7919 + 11)
    ways = 64
    u = torch.rand(tables, 4, generator=g, dtype=torch.float64)
    tabs = []
    for t in range(tables):
        rows = int(round(math.exp(math.log(1e4) + float(u[t, 0]) * (math.log(max_rows) - math.log(1e4)))))
        dim = (64, 128, 256)[min(2, int(float(u[t, 1]) * 3))]
        mean = math.exp(float(u[t, 2]) * math.log(100.0))
        alpha = 0.9 + 0.4 * float(u[t, 3])
        tabs.append(TableCfg(rows, dim, FP16, alpha, "poisson", mean, 0, 200))
    cfg = WorkloadCfg("hetero", tabs, batch=batch, ways=ways, steps=steps, seed=seed)
    cfg.cache_bytes = cache_bytes  # type: ignore[attr-defined]
    return cfg


def split_cache_budget(cfg: WorkloadCfg, lookups_per_table: List[int], cache_bytes: int) -> None:
    """Split `cache_bytes` over the tables in proportion to measured bandwidth
    (lookups x dim, the per-table term of the paper's Eq. 3 / Eq. 6); a table
    never gets more slots than rows, and what it cannot use is re-split among
    the others.  Sets cfg.tables[t].cache_slots (whole sets of cfg.ways)."""
    T = len(cfg.tables)
    esz = [4 if t.dtype == FP32 else 2 for t in cfg.tables]
    row_b = [cfg.tables[i].dim * esz[i] for i in range(T)]
    weight = [float(lookups_per_table[i]) * cfg.tables[i].dim for i in range(T)]
    slots = [0] * T
    open_ = set(range(T))
    budget = float(cache_bytes)
    while open_ and budget > 0:
        wsum = sum(weight[i] for i in open_)
        if wsum <= 0:
            break
        capped = []
        for i in open_:
            share = budget * weight[i] / wsum
            cap = (cfg.tables[i].rows // cfg.ways) * cfg.ways
            if share / row_b[i] >= cap:
                capped.append(i)
        if not capped:
            for i in open_:
                share = budget * weight[i] / wsum
                slots[i] = (int(share / row_b[i]) // cfg.ways) * cfg.ways
            break
        for i in capped:
            slots[i] = (cfg.tables[i].rows // cfg.ways) * cfg.ways
            budget -= slots[i] * row_b[i]
            open_.discard(i)
    for i in range(T):
        cfg.tables[i].cache_slots = slots[i]


def place_and_split_cache_budget(cfg: WorkloadCfg, lookups_per_table: List[int], cache_bytes: int,
                                 resident_fraction: float, hbm_bandwidth: float = 4e12,
                                 cached_bandwidth: float = 45e9) -> List[int]:
    """Size- and bandwidth-aware placement (the paper's embedding table assignment, Section
    5.6.1): `resident_fraction` of the HBM budget holds whole tables chosen by the library's
    solver for Eq. 6 (memory types: HBM at `hbm_bandwidth`, the cached host tier at
    `cached_bandwidth`; sizes = the tables' rows, traffic = lookups x row bytes) -- such a
    table gets as many cache slots as rows, so it never misses after the first touch; the
    rest of the budget is split over the other tables in proportion to lookups x dim.
    Returns the indices of the resident tables."""
    from . import placement
    T = len(cfg.tables)
    row_b = [t.dim * (4 if t.dtype == FP32 else 2) for t in cfg.tables]
    full = [-(-t.rows // cfg.ways) * cfg.ways for t in cfg.tables]  # slots that hold every row: S * W >= H
    size = [full[i] * row_b[i] for i in range(T)]
    traffic = [float(lookups_per_table[i]) * row_b[i] for i in range(T)]
    res = placement.plan(size, traffic, [int(cache_bytes * resident_fraction), sum(size)],
                         [hbm_bandwidth, cached_bandwidth])
    assert res is not None  # the cached tier holds everything
    resident = [i for i in range(T) if res[0][i] == 0]
    rest = [0 if i in resident else lookups_per_table[i] for i in range(T)]
    split_cache_budget(cfg, rest, cache_bytes - sum(size[i] for i in resident))
    for i in resident:
        cfg.tables[i].cache_slots = full[i]
    return resident


def config_capacity(seed: int = 3, tables: int = 8, rows: int = 1 << 26, batch: int = 65536,
                    cache_bytes: int = 8 << 30, steps: int = 500) -> WorkloadCfg:
    """8 tables x 64M rows x dim 128 fp16 behind an 8 GiB cache (64-way), batch
    65536, pooling Poisson(40), Zipf 1.05, 30 % of each batch re-drawn from the
    previous 4 batches."""
    ways = 64
    slots = ((cache_bytes // tables) // 256 // ways) * ways
    tabs = [TableCfg(rows, 128, FP16, 1.05, "poisson", 40, 1, 200, cache_slots=min(slots, (rows // ways) * ways))
            for _ in range(tables)]
    return WorkloadCfg("capacity", tabs, batch=batch, ways=ways, steps=steps, seed=seed,
                       reuse_frac=0.30, reuse_window=4)


def config_locality(alpha: Optional[float], cache_frac: float, seed: int = 4, rows: int = 100_000_000,
                    batch: int = 32768, steps: int = 100) -> WorkloadCfg:
    """1 table x 100M rows x dim 64 fp16, batch 32768, pooling 32; one point of
    the (index distribution, cache size) sweep."""
    ways = 64
    tabs = [TableCfg(rows, 64, FP16, alpha, "fixed", 32, cache_slots=_slots(rows, cache_frac, ways))]
    nm = "locality_%s_%g" % ("uniform" if alpha is None else "a%g" % alpha, cache_frac)
    return WorkloadCfg(nm, tabs, batch=batch, ways=ways, steps=steps, seed=seed)


# --------------------------------------------------------------------------------------
# index streams
# --------------------------------------------------------------------------------------

def _gen(seed: int, *stream: int, device="cpu") -> torch.Generator:
    s = seed & 0xFFFFFFFF
    for x in stream:
        s = (s * 1000003 + (x + 1) * 7919 + 12345) % ((1 << 61) - 1)
    return torch.Generator(device=device).manual_seed(s)


def zipf_ranks(n: int, rows: int, alpha: Optional[float], gen: torch.Generator, device="cpu") -> torch.Tensor:
    """n ranks in [0, rows): bounded power law with density ~ x^-alpha on
    [1, rows+1) drawn by inverting its CDF, floored (rank 0 is the hottest).
    alpha None = uniform.  Works for alpha below, at and above 1."""
    u = torch.rand(n, generator=gen, dtype=torch.float64, device=device)
    if alpha is None:
        r = torch.floor(u * rows)
    elif abs(alpha - 1.0) < 1e-12:
        r = torch.floor(torch.exp(u * math.log(rows + 1.0))) - 1.0
    else:
        e = 1.0 - alpha
        top = (rows + 1.0) ** e
        r = torch.floor(((top - 1.0) * u + 1.0) ** (1.0 / e)) - 1.0
    return r.clamp_(0, rows - 1).to(torch.int64)


class RankToRow:
    """Seeded bijection rank -> row id: an explicit random permutation for
    tables up to 10M rows, an affine map a*x + c (mod rows) with gcd(a, rows) = 1
    above that."""

    def __init__(self, rows: int, seed: int, table: int, device="cpu"):
        self.rows = rows
        g = _gen(seed, 101, table)
        if rows <= 10_000_000:
            self.perm = torch.randperm(rows, generator=g).to(device)
            self.a = self.c = None
        else:
            self.perm = None
            a = int(torch.randint(rows // 3, rows - 1, (1,), generator=g))
            while math.gcd(a, rows) != 1:
                a += 1
            self.a = a % rows
            self.c = int(torch.randint(0, rows, (1,), generator=g))

    def __call__(self, ranks: torch.Tensor) -> torch.Tensor:
        if self.perm is not None:
            return self.perm[ranks]
        # a, rank < rows <= 2^31-ish here, so the product fits int64
        return (ranks * self.a + self.c) % self.rows


class BatchStream:
    """Deterministic stream of (indices, offsets) batches for a workload.

    indices: int64[N] table-local row ids, bag-major inside a table,
    tables concatenated; offsets: int64[T*B + 1], bag t*B + b covers
    indices[offsets[t*B+b] : offsets[t*B+b+1]]."""

    def __init__(self, cfg: WorkloadCfg, device="cpu"):
        self.cfg = cfg
        self.device = device
        self.maps = [RankToRow(t.rows, cfg.seed, i, device) for i, t in enumerate(cfg.tables)]
        self.history: List[List[torch.Tensor]] = [[] for _ in cfg.tables]
        self.step = 0

    def _lengths(self, t: TableCfg, gen) -> torch.Tensor:
        B = self.cfg.batch
        if t.pool_kind == "fixed":
            return torch.full((B,), int(t.pool_mean), dtype=torch.int64, device=self.device)
        lam = torch.full((B,), float(t.pool_mean), dtype=torch.float64, device=self.device)
        return torch.poisson(lam, generator=gen).to(torch.int64).clamp_(t.pool_lo, t.pool_hi)

    def next(self) -> Tuple[torch.Tensor, torch.Tensor]:
        cfg = self.cfg
        self.step += 1
        idx_parts, len_parts = [], []
        for ti, t in enumerate(cfg.tables):
            gen = _gen(cfg.seed, 202, ti, self.step, device=self.device)
            lens = self._lengths(t, gen)
            n = int(lens.sum())
            rows = self.maps[ti](zipf_ranks(n, t.rows, t.alpha, gen, self.device))
            hist = self.history[ti]
            if cfg.reuse_frac > 0 and hist and n > 0:
                pool = torch.cat(hist)
                take = torch.rand(n, generator=gen, device=self.device) < cfg.reuse_frac
                pick = torch.randint(0, pool.numel(), (n,), generator=gen, device=self.device)
                rows = torch.where(take, pool[pick], rows)
            if cfg.reuse_frac > 0:
                hist.append(rows)
                if len(hist) > cfg.reuse_window:
                    hist.pop(0)
            idx_parts.append(rows)
            len_parts.append(lens)
        indices = torch.cat(idx_parts) if idx_parts else torch.zeros(0, dtype=torch.int64, device=self.device)
        lens = torch.cat(len_parts)
        offsets = torch.zeros(lens.numel() + 1, dtype=torch.int64, device=self.device)
        torch.cumsum(lens, 0, out=offsets[1:])
        return indices.contiguous(), offsets


def grad_out(cfg: WorkloadCfg, step: int, device="cpu") -> torch.Tensor:
    """Upstream gradient of the pooled output, N(0,1), fp32 [batch, sum_dim]."""
    g = _gen(cfg.seed, 303, step, device=device)
    return torch.randn(cfg.batch, cfg.sum_dim, generator=g, dtype=torch.float32, device=device)


def init_table(cfg: WorkloadCfg, t: int, device="cpu", chunk_rows: int = 1 << 22, out: torch.Tensor = None) -> torch.Tensor:
    """Initial weights of table t: N(0, init_std), fp32 or fp16 [rows, dim].
    Generated in chunks on `device`; written into `out` (any device, e.g. a
    pinned host tensor) when given."""
    tc = cfg.tables[t]
    dt = torch.float32 if tc.dtype == FP32 else torch.float16
    if out is None:
        out = torch.empty(tc.rows, tc.dim, dtype=dt, device=device)
    g = _gen(cfg.seed, 404, t, device=device)
    for r0 in range(0, tc.rows, chunk_rows):
        r1 = min(tc.rows, r0 + chunk_rows)
        blk = torch.randn(r1 - r0, tc.dim, generator=g, dtype=torch.float32, device=device) * cfg.init_std
        out[r0:r1].copy_(blk.to(dt))
    return out
