// Index dedup part 2 (run-length encoding of the sorted keys), the set-associative probe
// with LRU victim choice and miss-list compaction.  Paper Section 5.5: tag/state lookup
// (5.5.1, probe and grouping by destination) and cache algorithm (5.5.2), one-level cache.
#include "tbe_internal.h"

namespace tbe {

// --------------------------------------------------------------------------------------
// Generic flag -> exclusive prefix -> emit skeleton over n elements (n may live on the
// device).  Two 32-bit counters are scanned at once, packed into one 64-bit word.
//   count kernel : sum of op.flag(i) over the contiguous chunk of every wavefront, and per workgroup
//   emit kernel  : op.emit(i, exclusive prefix, flag) for every element, in order
// The unit is the wavefront: each one walks a chunk of its own and scans with lane shuffles only, so
// the emit pass has no barrier inside its loop -- a wave that waits for memory holds up nobody.  (With
// a workgroup-wide scan per tile, two barriers each, the waves of a workgroup ran at the pace of the
// slowest one, tile after tile: the emit passes of the benchmark workload took 0.11 ms each.)
// --------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanWavesPerBlock = kScanThreads / kWave;
// Consecutive elements per lane and step: Op::kItems.  With several, the lanes of one store instruction write
// compacted entries that lie apart (the entries of a lane's other elements fall between them), and the emit pass
// that flags a third of its elements and writes seven arrays wrote 121 MB for 32 MB of lists (49 us; 38 MB and
// 34 us with one element per lane); the passes that flag nearly every element or nearly none are faster with four.
#ifndef TBE_SCAN_BLOCKS
#define TBE_SCAN_BLOCKS 1024
#endif
constexpr int kScanBlocks = TBE_SCAN_BLOCKS;     // workgroups at most (SortScratch::blk holds 5 words per workgroup)

typedef unsigned long long u64;

__device__ inline u64 wave_incl_scan(u64 v, int lane) {
  for (int d = 1; d < 64; d <<= 1) {
    u64 o = __shfl_up(v, d);
    if (lane >= d) v += o;
  }
  return v;
}

__device__ inline u64 wave_total(u64 v) {
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// elements per wavefront: n spread over all wavefronts of the grid, in whole steps
__device__ inline int scan_chunk(int n, int nblocks, int step) {
  const int waves = nblocks * kScanWavesPerBlock;
  const int steps = (n + step - 1) / step;
  return (steps + waves - 1) / waves * step;
}

// blk: [0, nblocks) sums per workgroup; [nblocks, nblocks * 5) sums per wavefront
template <class Op>
__global__ __launch_bounds__(kScanThreads) void compact_count_kernel(Op op, const int32_t *n_ptr, int n_fixed,
                                                                     u64 *blk, const BatchCounters *cnt) {
  __shared__ u64 wsum[kScanWavesPerBlock];
  if (cnt->err) return;
  constexpr int kScanItems = Op::kItems, kScanStep = kWave * kScanItems;
  const int n = n_ptr ? *n_ptr : n_fixed;
  const int chunk = scan_chunk(n, gridDim.x, kScanStep);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int w = blockIdx.x * kScanWavesPerBlock + wave;
  const int64_t base64 = (int64_t)w * chunk;
  const int base = (int)(base64 < n ? base64 : n), end = (int)(base64 + chunk < n ? base64 + chunk : n);
  u64 s = 0;
  for (int i0 = base + lane * kScanItems; i0 < end; i0 += kScanStep) {
#pragma unroll
    for (int q = 0; q < kScanItems; q++)
      if (i0 + q < end) s += op.flag(i0 + q, n);
  }
  s = wave_total(s);
  if (lane == 0) {
    wsum[wave] = s;
    blk[gridDim.x + w] = s;
  }
  __syncthreads();
  if (tid == 0) {
    u64 t = 0;
    for (int k = 0; k < kScanWavesPerBlock; k++) t += wsum[k];
    blk[blockIdx.x] = t;
  }
}

// Per-table constants the emit passes need for every flagged element, copied to LDS by the workgroup (a
// look-up in the table descriptions in memory is a chain of dependent loads per element otherwise).
#ifndef TBE_FINALIZE_BLOCKS
#define TBE_FINALIZE_BLOCKS 512  // a multiple of 8
#endif
constexpr int kLutTables = 512;  // models with more tables read the descriptions from memory
struct TableLut {
  uint32_t key_base[kLutTables], sets[kLutTables], rows_per_set[kLutTables], set_base[kLutTables], row_bytes[kLutTables];
  char *host_w[kLutTables];
  char *lines2[kLutTables];
  int32_t slot2_base[kLutTables];
};

__device__ inline void fill_lut(TableLut &l, const TableMeta *tm, int T) {
  for (int t = threadIdx.x; t < T && t < kLutTables; t += blockDim.x) {
    l.key_base[t] = tm[t].key_base; l.sets[t] = tm[t].sets; l.rows_per_set[t] = tm[t].rows_per_set;
    l.set_base[t] = tm[t].set_base; l.row_bytes[t] = tm[t].row_bytes; l.host_w[t] = tm[t].host_w;
    l.lines2[t] = tm[t].lines2; l.slot2_base[t] = tm[t].slot2_base;
  }
}

template <class Op>
__global__ __launch_bounds__(kScanThreads) void compact_emit_kernel(Op op, const int32_t *n_ptr, int n_fixed,
                                                                    const u64 *blk, BatchCounters *cnt) {
  __shared__ TableLut s_lut;
  if (cnt->err) return;
  if (op.prepare(s_lut)) __syncthreads();
  constexpr int kScanItems = Op::kItems, kScanStep = kWave * kScanItems;
  const int n = n_ptr ? *n_ptr : n_fixed;
  const int chunk = scan_chunk(n, gridDim.x, kScanStep);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int w = blockIdx.x * kScanWavesPerBlock + wave;
  const int64_t base64 = (int64_t)w * chunk;
  const int base = (int)(base64 < n ? base64 : n), end = (int)(base64 + chunk < n ? base64 + chunk : n);
  // flags before this wavefront: the workgroups before its own, then the waves before it in its own
  u64 carry = 0;
  for (int b = lane; b < (int)blockIdx.x; b += kWave) carry += blk[b];
  if (lane < wave) carry += blk[gridDim.x + blockIdx.x * kScanWavesPerBlock + lane];
  carry = wave_total(carry);
  u64 total = 0;
  if (blockIdx.x == 0 && wave == 0) {
    for (int b = lane; b < (int)gridDim.x; b += kWave) total += blk[b];
    total = wave_total(total);
  }
  for (int i0 = base + lane * kScanItems; i0 - lane * kScanItems < end; i0 += kScanStep) {
    u64 f[kScanItems];
    u64 tsum = 0;
#pragma unroll
    for (int q = 0; q < kScanItems; q++) {
      f[q] = (i0 + q < end) ? op.flag(i0 + q, n) : 0;
      tsum += f[q];
    }
    const u64 incl = wave_incl_scan(tsum, lane);
    u64 pre = carry + incl - tsum;
#pragma unroll
    for (int q = 0; q < kScanItems; q++) {
      if (i0 + q < end) op.emit(i0 + q, n, pre, f[q]);
      pre += f[q];
    }
    carry += __shfl(incl, 63, 64);
  }
  op.thread_done(cnt, lane);
  if (blockIdx.x == 0 && tid == 0) op.finish(cnt, n, total);
}

// returns the number of workgroups of the two kernels
template <class Op>
static int run_compaction(Op op, const int32_t *n_ptr, int n_fixed, int n_bound, u64 *blk, BatchCounters *cnt,
                           hipStream_t s) {
  int nb = (n_bound + kScanThreads * Op::kItems - 1) / (kScanThreads * Op::kItems);
  if (nb > kScanBlocks) nb = kScanBlocks;
  if (nb < 1) nb = 1;
  hipLaunchKernelGGL(compact_count_kernel<Op>, dim3(nb), dim3(kScanThreads), 0, s, op, n_ptr, n_fixed, blk, cnt);
  hipLaunchKernelGGL(compact_emit_kernel<Op>, dim3(nb), dim3(kScanThreads), 0, s, op, n_ptr, n_fixed, blk, cnt);
  return nb;
}

// ---- pass 1 over the N sorted lookups: distinct rows, run starts, set ids ----
struct DedupOp {
  static constexpr int kItems = 2;
  const TableMeta *tm;
  int T;
  const uint32_t *key;      // sorted
  const uint32_t *pos;      // lookup position of each sorted element
  const int32_t *bag_of_pos;
  const BatchCounters *cnt;  // cnt->packed: the payload carries the bag
  int within_bits;
  const int64_t *offsets;
  int32_t *sorted_within;    // max pooling only (else null): position of the lookup inside its bag
  uint32_t *uid_sorted;
  int32_t *sorted_bag;
  uint32_t *uniq_key;
  int32_t *run_off;
  uint32_t *uniq_sid;
  int32_t *uniq_tab;
  mutable const TableLut *lut;  // null: the model has too many tables for it
  __device__ bool prepare(TableLut &l) const {
    lut = T <= kLutTables ? &l : nullptr;
    if (lut) fill_lut(l, tm, T);
    return lut != nullptr;
  }
  __device__ u64 flag(int i, int) const { return (i == 0 || key[i] != key[i - 1]) ? 1ull : 0ull; }
  __device__ void emit(int i, int, u64 pre, u64 f) const {
    const uint32_t u = (uint32_t)(pre & 0xFFFFFFFFull) + (uint32_t)f - 1u;
    uid_sorted[i] = u;
    const uint32_t p = pos[i];
    const int32_t bag = cnt->packed ? (int32_t)(p >> within_bits) : bag_of_pos[p];
    sorted_bag[i] = bag;
    if (sorted_within)
      sorted_within[i] = cnt->packed ? (int32_t)(p & ((1u << within_bits) - 1u)) : (int32_t)((int64_t)p - offsets[bag]);
    if (f) {
      const uint32_t k = key[i];
      uniq_key[u] = k;
      run_off[u] = i;
      if (lut) {
        int lo = 0, hi = T - 1;  // table that owns the key: last t with key_base[t] <= k
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (lut->key_base[mid] <= k) lo = mid; else hi = mid - 1;
        }
        uniq_tab[u] = lo;
        uniq_sid[u] = lut->sets[lo] ? lut->set_base[lo] + (k - lut->key_base[lo]) / lut->rows_per_set[lo] : kNoSet;
      } else {
        const int t = find_table(tm, T, k);
        const TableMeta &m = tm[t];
        uniq_tab[u] = t;
        uniq_sid[u] = m.sets ? m.set_base + (k - m.key_base) / m.rows_per_set : kNoSet;
      }
    }
  }
  __device__ void thread_done(BatchCounters *, int) const {}
  __device__ void finish(BatchCounters *cnt, int n, u64 total) const {
    cnt->n_uniq = (int32_t)(total & 0xFFFFFFFFull);
    run_off[total & 0xFFFFFFFFull] = n;
  }
};

// ---- pass 2 over the distinct rows: first row of every touched set; long runs ----
struct SetHeadOp {
  static constexpr int kItems = 4;
  const uint32_t *uniq_sid;
  const int32_t *run_off;
  uint2 *touched;
  __device__ bool prepare(TableLut &) const { return false; }
  __device__ u64 flag(int u, int) const { return (u == 0 || uniq_sid[u] != uniq_sid[u - 1]) ? 1ull : 0ull; }
  __device__ void emit(int u, int, u64 pre, u64 f) const {
    if (f) touched[pre & 0xFFFFFFFFull] = make_uint2(uniq_sid[u], (uint32_t)u);
  }
  __device__ void thread_done(BatchCounters *, int) const {}
  __device__ void finish(BatchCounters *cnt, int, u64 total) const { cnt->n_touched = (int32_t)(total & 0xFFFFFFFFull); }
};

// Work lists of the backward by run length (see kLongRun), in the order of the distinct rows (= table
// order: the backward kernels give each XCD a contiguous part of a list).  A workgroup takes a contiguous
// chunk of the distinct rows; the count kernel leaves the two counts of every workgroup in `wl`, the
// emit kernel adds up the counts of the workgroups before it and writes its rows out in order.  It also
// counts the heavy rows of every table.
__device__ inline void worklist_chunk(int n, int &w0, int &w1) {
  const int wave = threadIdx.x >> 6;
  const int per_wave = ((n + gridDim.x * 4 - 1) / (gridDim.x * 4) + 63) / 64 * 64;
  w0 = (blockIdx.x * 4 + wave) * per_wave;
  w1 = min(n, w0 + per_wave);
}

__device__ inline int wave_sum(int v) {
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// counts of the wavefront's chunk: (rows with 2..kLongRun lookups, heavy-list entries of the rows with more)
__device__ inline void worklist_tally(const int32_t *__restrict__ run_off, int w0, int w1, int (&c)[2]) {
  const int lane = threadIdx.x & 63;
  c[0] = c[1] = 0;
  for (int u0 = w0; u0 < w1; u0 += 64) {
    const int u = u0 + lane;
    const int len = u < w1 ? run_off[u + 1] - run_off[u] : 0;
    c[0] += __popcll(__ballot(len >= 2 && len <= kLongRun));
    if (__ballot(len > kLongRun)) c[1] += wave_sum(len > kLongRun ? heavy_parts(len) : 0);
  }
}

__global__ __launch_bounds__(256) void worklist_count_kernel(const int32_t *__restrict__ run_off, int32_t *wl,
                                                             const BatchCounters *cnt) {
  __shared__ int s_cnt[4][2];
  if (cnt->err) return;
  int w0, w1, c[2];
  worklist_chunk(cnt->n_uniq, w0, w1);
  worklist_tally(run_off, w0, w1, c);
  if ((threadIdx.x & 63) == 0)
    for (int k = 0; k < 2; k++) s_cnt[threadIdx.x >> 6][k] = c[k];
  __syncthreads();
  if (threadIdx.x < 2) wl[blockIdx.x * 2 + threadIdx.x] = s_cnt[0][threadIdx.x] + s_cnt[1][threadIdx.x] + s_cnt[2][threadIdx.x] + s_cnt[3][threadIdx.x];
}

__global__ __launch_bounds__(256) void worklist_emit_kernel(const int32_t *__restrict__ run_off,
                                                            const int32_t *__restrict__ uniq_tab,
                                                            const int32_t *__restrict__ wl, int32_t *mid_idx,
                                                            int32_t *heavy, int32_t *heavy_sub,
                                                            int32_t *heavy_per_table, BatchCounters *cnt) {
  __shared__ int s_cnt[4][2];
  __shared__ int s_before[4][2];
  __shared__ int s_base[4][2];
  // Heavy-list entries per table: gathered in LDS for the tables this workgroup's rows belong to (its rows are
  // consecutive, so these are few) and added to the totals once per table -- thousands of atomic additions
  // from all over the chip to a few dozen addresses took ten times as long as the rest of this kernel.
  constexpr int kLocalTables = 256;
  __shared__ int s_tab[kLocalTables];
  __shared__ int s_tab0;
  if (cnt->err) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  int w0, w1, c[2];
  worklist_chunk(cnt->n_uniq, w0, w1);
  s_tab[threadIdx.x] = 0;
  if (threadIdx.x == 0) {
    int b0, b1;
    worklist_chunk(cnt->n_uniq, b0, b1);  // wave 0: the workgroup's first row
    s_tab0 = b0 < cnt->n_uniq ? uniq_tab[b0] : 0;
  }
  worklist_tally(run_off, w0, w1, c);
  int before[2] = {0, 0};  // rows of each kind in the workgroups before this one
  for (int b = threadIdx.x; b < (int)blockIdx.x; b += 256)
    for (int k = 0; k < 2; k++) before[k] += wl[b * 2 + k];
  for (int k = 0; k < 2; k++)
    for (int d = 32; d >= 1; d >>= 1) before[k] += __shfl_xor(before[k], d, 64);
  if (lane == 0)
    for (int k = 0; k < 2; k++) { s_cnt[wave][k] = c[k]; s_before[wave][k] = before[k]; }
  __syncthreads();
  if (threadIdx.x < 2) {
    const int k = threadIdx.x;
    int base = s_before[0][k] + s_before[1][k] + s_before[2][k] + s_before[3][k];
    for (int w = 0; w < 4; w++) { s_base[w][k] = base; base += s_cnt[w][k]; }
    if (blockIdx.x == gridDim.x - 1) {  // the last workgroup knows the totals
      if (k == 0) cnt->n_mid = base;
      if (k == 1) cnt->n_heavy = base;
    }
  }
  __syncthreads();
  int o_mid = s_base[wave][0], o_heavy = s_base[wave][1];
  for (int u0 = w0; u0 < w1; u0 += 64) {
    const int u = u0 + lane;
    const int len = u < w1 ? run_off[u + 1] - run_off[u] : 0;
    const bool is_mid = len >= 2 && len <= kLongRun;
    const bool is_heavy = len > kLongRun;
    const uint64_t bm = __ballot(is_mid);
    if (is_mid) mid_idx[o_mid + __popcll(bm & lt_mask)] = u;
    o_mid += __popcll(bm);
    if (__ballot(is_heavy)) {  // uniform: the entries of the wavefront's heavy rows, in row order
      const int parts = is_heavy ? heavy_parts(len) : 0;
      int incl = parts;
      for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
      }
      const int at = o_heavy + incl - parts;
      for (int q = 0; q < parts; q++) {
        heavy[at + q] = u;
        heavy_sub[at + q] = q | (parts << 16);
      }
      if (is_heavy) {
        const int t = uniq_tab[u], rel = t - s_tab0;
        if (rel >= 0 && rel < kLocalTables) atomicAdd(&s_tab[rel], parts); else atomicAdd(&heavy_per_table[t], parts);
      }
      o_heavy += __shfl(incl, 63, 64);
    }
  }
  __syncthreads();
  if (s_tab[threadIdx.x]) atomicAdd(&heavy_per_table[s_tab0 + threadIdx.x], s_tab[threadIdx.x]);
}

// The heavy list is in table order.  Cut every table's part into chunks of the rows one workgroup of the
// tile kernel takes (heavy_chunk_rows of the table's lanes per row), and fix the number of bag ranges of
// this batch.  One workgroup; tables are taken 256 at a time.
__global__ __launch_bounds__(256) void heavy_group_kernel(const TableMeta *__restrict__ tm, int T,
                                                          const int32_t *__restrict__ heavy_per_table,
                                                          int32_t *first_of_table, uint4 *hchunks,
                                                          long long slot_capacity, int target_items,
                                                          BatchCounters *cnt) {
  __shared__ int s_rows[4], s_chunks[4];
  __shared__ int s_carry[2];
  if (cnt->err) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) s_carry[0] = s_carry[1] = 0;
  __syncthreads();
  for (int t0 = 0; t0 < T; t0 += 256) {
    const int t = t0 + tid;
    const int rows = t < T ? heavy_per_table[t] : 0;
    const int per = t < T ? heavy_chunk_rows(tm[t].lanes, tm[t].dtype) : 1;
    const int chunks = (rows + per - 1) / per;
    int ir = rows, ic = chunks;  // inclusive scans over the workgroup
    for (int d = 1; d < 64; d <<= 1) {
      const int a = __shfl_up(ir, d), b = __shfl_up(ic, d);
      if (lane >= d) { ir += a; ic += b; }
    }
    if (lane == 63) { s_rows[wave] = ir; s_chunks[wave] = ic; }
    __syncthreads();
    int row0 = s_carry[0] + ir - rows, chunk0 = s_carry[1] + ic - chunks;
    for (int w = 0; w < wave; w++) { row0 += s_rows[w]; chunk0 += s_chunks[w]; }
    if (t < T) first_of_table[t] = row0;
    for (int c = 0; c < chunks; c++)
      hchunks[chunk0 + c] = make_uint4((uint32_t)t, (uint32_t)(row0 + c * per), (uint32_t)min(per, rows - c * per), 0u);
    __syncthreads();
    if (tid == 255) { s_carry[0] = row0 + rows; s_carry[1] = chunk0 + chunks; }
    __syncthreads();
  }
  if (tid == 0) {
    cnt->n_hchunks = s_carry[1];
    cnt->h_ranges = heavy_ranges(s_carry[1], cnt->n_heavy, slot_capacity, target_items);
  }
}

// Order of a table's heavy-list entries for the tile kernel: by lookups per entry, descending, in classes of
// powers of two (entries of a class keep their order, so the result is a function of the batch alone).  The
// tile kernel deals the entries round its lane groups in this order, so the groups that share a wavefront --
// which runs as long as its busiest group -- get rows of like length.  One wavefront per table.
__global__ __launch_bounds__(64) void heavy_order_kernel(const int32_t *__restrict__ heavy_per_table,
                                                         const int32_t *__restrict__ first_of_table,
                                                         const int32_t *__restrict__ heavy,
                                                         const int32_t *__restrict__ heavy_sub,
                                                         const int32_t *__restrict__ run_off, int32_t *hperm,
                                                         const BatchCounters *cnt) {
  __shared__ int s_base[32];
  if (cnt->err) return;
  const int t = blockIdx.x, lane = threadIdx.x;
  const int n = heavy_per_table[t], first = first_of_table[t];
  if (n == 0) return;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  auto klass = [&](int h) {  // 31 - floor(log2(lookups per entry)): longer entries first
    const int u = heavy[h];
    const int len = (run_off[u + 1] - run_off[u]) / (heavy_sub[h] >> 16);
    return __clz(len < 1 ? 1 : len);
  };
  if (lane < 32) s_base[lane] = 0;
  __syncthreads();
  for (int i0 = 0; i0 < n; i0 += 64)
    if (i0 + lane < n) atomicAdd(&s_base[klass(first + i0 + lane)], 1);
  __syncthreads();
  if (lane == 0) {
    int at = 0;
    for (int k = 0; k < 32; k++) { const int c = s_base[k]; s_base[k] = at; at += c; }
  }
  __syncthreads();
  for (int i0 = 0; i0 < n; i0 += 64) {
    const bool valid = i0 + lane < n;
    const int k = valid ? klass(first + i0 + lane) : -1;
    uint64_t todo = __ballot(valid);
    while (todo) {  // one class at a time, its entries in order
      const int kk = __shfl(k, __ffsll((unsigned long long)todo) - 1, 64);
      const uint64_t same = __ballot(k == kk);
      if (k == kk) hperm[first + s_base[kk] + __popcll(same & lt_mask)] = first + i0 + lane;
      __syncthreads();
      if (lane == 0) s_base[kk] += __popcll(same);
      __syncthreads();
      todo &= ~same;
    }
  }
}

// For every entry of the heavy list and bag range: the first sorted position of the entry's row whose bag
// lies in the range (the row's lookups are sorted by bag).  One thread per (entry, range).
__global__ __launch_bounds__(256) void heavy_starts_kernel(const TableMeta *__restrict__ tm, int B,
                                                           const int32_t *__restrict__ heavy,
                                                           const int32_t *__restrict__ uniq_tab,
                                                           const int32_t *__restrict__ run_off,
                                                           const int32_t *__restrict__ sorted_bag, int32_t *hstart,
                                                           const BatchCounters *cnt) {
  if (cnt->err) return;
  const int R = cnt->h_ranges;
  const int n = cnt->n_heavy * R;
  for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < n; x += gridDim.x * blockDim.x) {
    const int h = x / R, range = x % R;
    const int u = heavy[h];
    const int t = uniq_tab[u];
    const long long first_bag = (long long)t * B + heavy_range_first(B, R, range);
    int lo = run_off[u], hi = run_off[u + 1];
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sorted_bag[mid] < first_bag) lo = mid + 1; else hi = mid;
    }
    hstart[x] = lo;
  }
}

// ---- pass 3 over the distinct rows after the probe: insert and bypass lists, counters ----
struct StatusOp {
  static constexpr int kItems = 1;
  const TableMeta *tm;
  int T;
  const uint8_t *status;
  const int32_t *run_off;
  const int32_t *old_tag;
  const uint32_t *uniq_key;
  const int32_t *uniq_tab;
  int32_t *ins_idx;
  int32_t *ins_tab;
  int32_t *ins_slot;
  int32_t *ins_old;
  uint32_t *ins_key;
  char **ins_src;
  int32_t *byp_idx;
  int32_t *byp_tab;
  uint32_t *byp_key;
  char **byp_src;
  int32_t *loc_u;
  // second level (all null without one)
  const int32_t *src2, *dst2, *evict2;
  char **ins_dst, **l2v_src, **l2v_dst;
  uint32_t *l2v_key;
  // per-thread tallies (the emit kernel keeps one Op copy per thread in registers); every wavefront leaves
  // its sums in `tally` (two words each), which the kernel that keeps the running totals adds up -- thousands
  // of atomic additions to one counter from all over the chip would take longer than the pass itself
  u64 *tally;
  mutable unsigned int evs;
  mutable u64 hit_lookups;
  mutable const TableLut *lut;  // null: the model has too many tables for it
  __device__ bool prepare(TableLut &l) const {
    lut = T <= kLutTables ? &l : nullptr;
    if (lut) fill_lut(l, tm, T);
    return lut != nullptr;
  }
  struct TabView {
    uint32_t key_base, sets, rows_per_set, row_bytes;
    char *host_w, *lines2;
    int32_t slot2_base;
    __device__ uint32_t row_of(uint32_t key) const {
      const uint32_t local = key - key_base;
      if (sets == 0) return local;
      const uint32_t s = local / rows_per_set;
      return (local - s * rows_per_set) * sets + s;
    }
    __device__ uint32_t key_of(uint32_t row) const {
      if (sets == 0) return key_base + row;
      const uint32_t q = row / sets;
      return key_base + (row - q * sets) * rows_per_set + q;
    }
  };
  __device__ TabView view(int t) const {
    if (lut)
      return TabView{lut->key_base[t], lut->sets[t], lut->rows_per_set[t], lut->row_bytes[t], lut->host_w[t], lut->lines2[t],
                     lut->slot2_base[t]};
    const TableMeta &m = tm[t];
    return TabView{m.key_base, m.sets, m.rows_per_set, m.row_bytes, m.host_w, m.lines2, m.slot2_base};
  }
  __device__ u64 flag(int u, int) const {
    const uint8_t s = status[u];
    return s == ST_INSERT ? 1ull : s == ST_BYPASS ? (1ull << 32) : 0ull;
  }
  __device__ void emit(int u, int, u64 pre, u64 f) const {
    if (f == 1ull) {
      const uint32_t i = (uint32_t)(pre & 0xFFFFFFFFull);
      const uint32_t key = uniq_key[u];
      const int t = uniq_tab[u];
      const TabView m = view(t);
      const uint32_t row = m.row_of(key);
      const int32_t old = old_tag[u];
      ins_idx[i] = u;
      ins_tab[i] = t;
      ins_slot[i] = loc_u[u];
      ins_old[i] = old;
      ins_key[i] = key;
      ins_src[i] = m.host_w + (size_t)row * m.row_bytes;
      if (src2) {  // second level: the row may come from there, the victim may go there
        const int32_t s2 = src2[u], d2 = dst2[u], e2 = evict2[u];
        if (s2 >= 0) ins_src[i] = m.lines2 + (size_t)(s2 - m.slot2_base) * m.row_bytes;
        char *dst = old >= 0 ? m.host_w + (size_t)old * m.row_bytes : nullptr;
        if (old >= 0 && d2 >= 0) dst = m.lines2 + (size_t)(d2 - m.slot2_base) * m.row_bytes;
        ins_dst[i] = dst;
        l2v_src[i] = e2 >= 0 ? dst : nullptr;  // the line the victim takes still holds the row it pushes out
        l2v_dst[i] = e2 >= 0 ? m.host_w + (size_t)e2 * m.row_bytes : nullptr;
        l2v_key[i] = e2 >= 0 ? m.key_of((uint32_t)e2) : 0u;
      }
      if (old >= 0) evs++;
    } else if (f) {
      const uint32_t j = (uint32_t)(pre >> 32);
      const uint32_t key = uniq_key[u];
      const int t = uniq_tab[u];
      const TabView m = view(t);
      byp_idx[j] = u;
      byp_tab[j] = t;
      byp_key[j] = key;
      byp_src[j] = m.host_w + (size_t)m.row_of(key) * m.row_bytes;
      if (src2 && src2[u] >= 0)  // lives in the second level: used in place
        byp_src[j] = m.lines2 + (size_t)(src2[u] - m.slot2_base) * m.row_bytes;
      loc_u[u] = -2 - (int32_t)j;  // the row is served from the j-th overflow slot
    } else if (status[u] == ST_HIT) {
      hit_lookups += (u64)(run_off[u + 1] - run_off[u]);
    }
  }
  __device__ void thread_done(BatchCounters *, int lane) const {
    u64 e = evs, l = hit_lookups;
    for (int d = 32; d >= 1; d >>= 1) {
      e += __shfl_xor(e, d);
      l += __shfl_xor(l, d);
    }
    if (lane == 0) {
      const int w = blockIdx.x * kScanWavesPerBlock + (threadIdx.x >> 6);
      tally[2 * w] = e;
      tally[2 * w + 1] = l;
    }
  }
  __device__ void finish(BatchCounters *cnt, int, u64 total) const {
    cnt->n_ins = (int32_t)(total & 0xFFFFFFFFull);
    cnt->n_byp = (int32_t)(total >> 32);
  }
};

// --------------------------------------------------------------------------------------
// Probe + replacement.  A wavefront takes a window of consecutive touched sets -- as many as hold about a
// wavefront's width of distinct rows, at most kProbeSets -- and keeps the ways of all of them in LDS.
//   phase 1, a lane per distinct row over the whole window: a row that is found is a hit, its way is
//            stamped k and its count grows by the row's lookups in the batch;
//   phase 2, per set of the window that has a miss, lane w holding way w: the evictable ways are ranked by
//            (timestamp, way) -- LRU -- or by (count, timestamp, way) -- LFU; the j-th miss in ascending
//            row order takes the way of rank j (evicting what it held) and starts counting at its own
//            lookups; misses beyond the number of such ways bypass the cache.
// Rows of a set arrive in ascending order because the sort key is (set, row div S).
// A set's chain of dependent reads (set head -> table -> ways -> rows) is several memory round trips; with a
// cache as large as the tables a batch touches a million sets with two or three rows each, and one set per
// wavefront left the kernel waiting on that chain (0.67 ms for the benchmark shapes with every row resident).
// --------------------------------------------------------------------------------------
__device__ inline int32_t add_saturating(int32_t a, int32_t b) {  // a, b >= 0
  const uint32_t v = (uint32_t)a + (uint32_t)b;
  return v > 0x7FFFFFFFu ? 0x7FFFFFFF : (int32_t)v;
}

#ifndef TBE_PROBE_SETS
#define TBE_PROBE_SETS 8
#endif
constexpr int kProbeSets = TBE_PROBE_SETS;       // sets of one window, at most
static_assert(TBE_PROBE_SETS >= 2 && TBE_PROBE_SETS <= 32, "a window's sets with a miss are a 32-bit mask; 32 ways per set of room make a set of 64 ways fit");
constexpr int kProbeWays = 32 * TBE_PROBE_SETS;  // ways of one window, at most (>= kWave, so that a window holds a set at least)
#ifndef TBE_PROBE_ROWS
#define TBE_PROBE_ROWS 64        // distinct rows a window aims for
#endif

template <bool LFU, bool L2>
__global__ __launch_bounds__(kWave) void probe_kernel(const TableMeta *__restrict__ tm, int T, int W, int32_t k,
                                                      int32_t evictable_below, int32_t min_windows,
                                                      const uint32_t *__restrict__ uniq_key,
                                                      const int32_t *__restrict__ uniq_tab,
                                                      const uint2 *__restrict__ touched, int32_t *__restrict__ tags,
                                                      int32_t *__restrict__ ts, int32_t *__restrict__ freq,
                                                      const int32_t *__restrict__ run_off,
                                                      int32_t *__restrict__ loc_u, uint8_t *__restrict__ status,
                                                      int32_t *__restrict__ old_tag, int32_t *__restrict__ tags2,
                                                      int32_t *__restrict__ ts2, int l2_factor,
                                                      int32_t *__restrict__ src2, int32_t *__restrict__ dst2,
                                                      int32_t *__restrict__ evict2, BatchCounters *cnt) {
  // ways of set i of the window at [i * (W + 1), i * (W + 1) + W): the odd stride keeps lanes that scan
  // different sets on different banks
  __shared__ int32_t w_tag[kProbeWays + kProbeSets], w_ts[kProbeWays + kProbeSets], w_freq[kProbeWays + kProbeSets];
  __shared__ int32_t h_u0[kProbeSets + 1], h_tab[kProbeSets], h_slot0[kProbeSets];
  __shared__ uint32_t h_key0[kProbeSets], h_sets[kProbeSets], h_set[kProbeSets];
  __shared__ int32_t l_way[kWave];
  __shared__ int32_t l_tag2[L2 ? kWave : 1], l_ts2[L2 ? kWave : 1], l_way2[L2 ? kWave : 1];
  __shared__ int32_t v_row[L2 ? kWave : 1], v_u[L2 ? kWave : 1];
  int n_l2hit = 0, n_l2dem = 0, n_l2ev = 0, n_l2byp = 0;  // this lane's share of the second-level counters
  if (cnt->err) return;
  const int lane = threadIdx.x;
  const int n_touched = cnt->n_touched, n_uniq = cnt->n_uniq;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const int WP = W + 1;
  int ns = n_uniq > 0 ? (int)(((long long)TBE_PROBE_ROWS * n_touched + n_uniq - 1) / n_uniq) : 1;
  int ns_max = kProbeWays / W < kProbeSets ? kProbeWays / W : kProbeSets;
  if (ns_max > n_touched / min_windows) ns_max = n_touched / min_windows;  // few sets: a wavefront each
  ns = ns > ns_max ? ns_max : ns;
  ns = ns < 1 ? 1 : ns;
  for (long long v0 = (long long)blockIdx.x * ns; v0 < n_touched; v0 += (long long)gridDim.x * ns) {
    const int nv = n_touched - v0 < ns ? (int)(n_touched - v0) : ns;
    __syncthreads();
    if (lane <= nv) {
      const long long v = v0 + lane;
      uint2 head = make_uint2(kNoSet, (uint32_t)n_uniq);
      if (v < n_touched) head = touched[v];
      h_u0[lane] = (int)head.y;
      if (lane < nv) {
        if (head.x == kNoSet) {  // rows of tables without a cache
          h_slot0[lane] = -1;
        } else {
          const int t = uniq_tab[head.y];
          const TableMeta &m = tm[t];
          const uint32_t set = head.x - m.set_base;
          h_tab[lane] = t;
          h_slot0[lane] = (int)head.x * W;  // global slot id of way 0 (set_base * W == slot_base)
          h_set[lane] = set;
          h_sets[lane] = m.sets;
          h_key0[lane] = m.key_base + set * m.rows_per_set;
        }
      }
    }
    __syncthreads();
    const int U0 = h_u0[0], U1 = h_u0[nv];
    for (int e = lane; e < nv * W; e += kWave) {
      const int si = e / W, w = e - si * W;
      const int s0 = h_slot0[si];
      if (s0 >= 0) {
        w_tag[si * WP + w] = tags[s0 + w];
        w_ts[si * WP + w] = ts[s0 + w];
        w_freq[si * WP + w] = freq[s0 + w];
      }
    }
    __syncthreads();
    // phase 1: hits, a lane per distinct row of the window
    uint32_t miss_sets = 0;
    for (int c = U0; c < U1; c += kWave) {
      const int u = c + lane;
      if (u < U1) {
        int si = 0;
        for (int i = 1; i < nv; i++) si += h_u0[i] <= u ? 1 : 0;
        const int s0 = h_slot0[si];
        if (L2) src2[u] = dst2[u] = evict2[u] = -1;
        if (s0 < 0) {
          loc_u[u] = -1;
          status[u] = ST_BYPASS;
        } else {
          const int32_t row = (int32_t)((uniq_key[u] - h_key0[si]) * h_sets[si] + h_set[si]);
          const int base = si * WP;
          int hit = -1;
          for (int w = 0; w < W; w++)
            if (w_tag[base + w] == row) hit = w;
          if (hit >= 0) {
            w_ts[base + hit] = k;
            w_freq[base + hit] = add_saturating(w_freq[base + hit], run_off[u + 1] - run_off[u]);
            loc_u[u] = s0 + hit;
            status[u] = ST_HIT;
          } else {
            status[u] = ST_MISS;
            miss_sets |= 1u << si;
          }
        }
      }
    }
    for (int d = 32; d >= 1; d >>= 1) miss_sets |= __shfl_xor(miss_sets, d);
    const uint32_t new_tags = miss_sets;  // only a miss changes a set's tags
    __syncthreads();
    while (miss_sets) {  // the same in every lane
      const int si = __ffs(miss_sets) - 1;
      miss_sets &= miss_sets - 1;
      const int base = si * WP;
      int32_t *l_tag = w_tag + base, *l_ts = w_ts + base, *l_freq = w_freq + base;
      const int u0 = h_u0[si], u1 = h_u0[si + 1];
      const int slot0 = h_slot0[si];
      const TableMeta &m = tm[h_tab[si]];
      const uint32_t set = h_set[si], key0 = h_key0[si];
      // phase 2: rank the evictable ways
      const int32_t my_ts = lane < W ? l_ts[lane] : 0x7FFFFFFF;
      // evictable: free ways (-1) and ways stamped before evictable_below = max(k - lock, 1): the ways of this batch
      // and, in a pipeline `lock` batches deep, of the batches that may still be waiting for their training
      const bool cand = lane < W && my_ts < evictable_below;
      const int32_t my_freq = lane < W ? l_freq[lane] : 0;
      int rank = 0;
      for (int w = 0; w < W; w++) {
        const int32_t tw = l_ts[w];
        if (tw >= evictable_below) continue;
        bool first = tw < my_ts || (tw == my_ts && w < lane);
        if (LFU) {
          const int32_t fw = l_freq[w];
          first = fw < my_freq || (fw == my_freq && first);
        }
        if (first) rank++;
      }
      const int n_cand = __popcll(__ballot(cand));
      __syncthreads();
      if (cand) l_way[rank] = lane;
      __syncthreads();
      int before = 0;
      for (int c = u0; c < u1; c += kWave) {
        const int u = c + lane;
        const bool miss = u < u1 && status[u] == ST_MISS;
        const uint64_t mb = __ballot(miss);
        if (miss) {
          const int j = before + __popcll(mb & lt_mask);
          if (j < n_cand) {
            const int way = l_way[j];
            old_tag[u] = l_tag[way];
            l_tag[way] = (int32_t)((uniq_key[u] - key0) * m.sets + set);
            l_ts[way] = k;
            l_freq[way] = run_off[u + 1] - run_off[u];
            loc_u[u] = slot0 + way;
            status[u] = ST_INSERT;
          } else {
            loc_u[u] = -1;
            status[u] = ST_BYPASS;
          }
        }
        before += __popcll(mb);
      }
      __syncthreads();
      if (L2) {
        // ---- second level (exclusive): the rows this set missed are looked up there, then the
        // rows this set evicted move down.  sets2 = l2_factor * sets, so a row r of this set
        // belongs to second-level set  set + sets * ((r div sets) mod l2_factor)  and no other
        // first-level set shares it: this wavefront owns all of them.
        int n_v = 0;  // the victims of this set: at most W, one per lane
        for (int c = u0; c < u1; c += kWave) {
          const int u = c + lane;
          const bool valid = u < u1;
          const bool isv = valid && status[u] == ST_INSERT && old_tag[u] >= 0;
          const uint64_t vm = __ballot(isv);
          if (isv) {
            const int p = n_v + __popcll(vm & lt_mask);
            v_row[p] = old_tag[u];
            v_u[p] = u;
          }
          n_v += __popcll(vm);
        }
        __syncthreads();
        const int32_t my_v = lane < n_v ? v_row[lane] : -1;
        const int my_vset = my_v >= 0 ? (int)(((uint32_t)my_v / m.sets) % (uint32_t)l2_factor) : -1;
        for (int j = 0; j < l2_factor; j++) {
          const int slot20 = m.slot2_base + (int)(set + (uint32_t)j * m.sets) * W;
          l_tag2[lane] = lane < W ? tags2[slot20 + lane] : -2;
          l_ts2[lane] = lane < W ? ts2[slot20 + lane] : 0x7FFFFFFF;
          __syncthreads();
          // (A) missed rows of this second-level set: found and inserted above -> moves up, its entry
          // becomes free; found but bypassed above -> stays, used in place, stamped k
          for (int c = u0; c < u1; c += kWave) {
            const int u = c + lane;
            const uint32_t q = u < u1 ? uniq_key[u] - key0 : 0u;  // row div sets
            const bool mine = u < u1 && status[u] != ST_HIT && (int)(q % (uint32_t)l2_factor) == j;
            const int32_t row = mine ? (int32_t)(q * m.sets + set) : -3;
            int hw = -1;
            for (int w = 0; w < W; w++)
              if (l_tag2[w] == row) hw = w;
            if (hw >= 0) {
              src2[u] = slot20 + hw;
              if (status[u] == ST_INSERT) { l_tag2[hw] = -1; l_ts2[hw] = -1; } else l_ts2[hw] = k;
              n_l2hit++;
            }
          }
          __syncthreads();
          // (B) victims of this second-level set in ascending row order take the ways older than
          // k - 1 in order of (timestamp, way); entries of this batch and the one before stay
          const bool vmine = my_vset == j;
          int vrank = 0;
          for (int w = 0; w < n_v; w++) {
            const int32_t o = v_row[w];
            if ((int)(((uint32_t)o / m.sets) % (uint32_t)l2_factor) == j && o < my_v) vrank++;
          }
          const int32_t my_ts2 = l_ts2[lane];
          const bool cand2 = lane < W && my_ts2 < k - 1;
          int rank2 = 0;
          for (int w = 0; w < W; w++) {
            const int32_t tw = l_ts2[w];
            if (tw < k - 1 && (tw < my_ts2 || (tw == my_ts2 && w < lane))) rank2++;
          }
          const int n_cand2 = __popcll(__ballot(cand2));
          if (cand2) l_way2[rank2] = lane;
          __syncthreads();
          if (vmine) {
            if (vrank < n_cand2) {
              const int way = l_way2[vrank];
              const int32_t held = l_tag2[way];
              evict2[v_u[lane]] = held;
              dst2[v_u[lane]] = slot20 + way;
              l_tag2[way] = my_v;
              l_ts2[way] = k;
              n_l2dem++;
              if (held >= 0) n_l2ev++;
            } else {
              n_l2byp++;  // no way to take: the victim goes to the lower tier
            }
          }
          __syncthreads();
          if (lane < W) {
            tags2[slot20 + lane] = l_tag2[lane];
            ts2[slot20 + lane] = l_ts2[lane];
          }
          __syncthreads();
        }
      }
    }
    __syncthreads();
    for (int e = lane; e < nv * W; e += kWave) {
      const int si = e / W, w = e - si * W;
      const int s0 = h_slot0[si];
      if (s0 >= 0) {
        if (new_tags >> si & 1u) tags[s0 + w] = w_tag[si * WP + w];
        ts[s0 + w] = w_ts[si * WP + w];
        freq[s0 + w] = w_freq[si * WP + w];
      }
    }
  }
  if (L2) {
    for (int d = 32; d >= 1; d >>= 1) {
      n_l2hit += __shfl_xor(n_l2hit, d); n_l2dem += __shfl_xor(n_l2dem, d);
      n_l2ev += __shfl_xor(n_l2ev, d); n_l2byp += __shfl_xor(n_l2byp, d);
    }
    if (lane == 0) {
      if (n_l2hit) atomicAdd(&cnt->l2_hits, n_l2hit);
      if (n_l2dem) atomicAdd(&cnt->l2_demotions, n_l2dem);
      if (n_l2ev) atomicAdd(&cnt->l2_evictions, n_l2ev);
      if (n_l2byp) atomicAdd(&cnt->l2_bypasses, n_l2byp);
    }
  }
}

// Per-lookup location word, in input order, written from the sorted side: lookup i of the sorted sequence
// belongs to distinct row uid_sorted[i], whose word goes to the lookup's position.  These are 4-byte stores all
// over the array, but not without order: the sorted sequence and the input are both table-major, so the words
// of one table land in that table's stretch of the array (a megabyte in the benchmark workload).  Each XCD takes
// a contiguous eighth of the sorted sequence, i.e. whole tables, so a table's stretch is written through one L2,
// where the stores meet and leave as full lines; the streamed inputs are read around the cache.  (Workgroups
// dealt round robin over the XCDs wrote every line from eight L2s, in eight partial pieces: 260 MB of write
// traffic for 31 MB of words.)
__global__ __launch_bounds__(256) void finalize_kernel(int n, const uint32_t *__restrict__ pos,
                                                       const uint32_t *__restrict__ uid_sorted,
                                                       const int32_t *__restrict__ loc_u,
                                                       const int32_t *__restrict__ run_off, uint32_t *__restrict__ loc,
                                                       const int64_t *__restrict__ offsets, int within_bits,
                                                       const BatchCounters *cnt) {
  if (cnt->err) return;
  const bool packed = cnt->packed != 0;
  const uint32_t within_mask = (1u << within_bits) - 1u;
  constexpr int K = 4;  // lookups per thread and pass, a workgroup's width apart: their loads are in flight together
  int first, end, step;
  xcd_span(n, 256 * K, first, end, step);
  for (int i0 = first + threadIdx.x; i0 < end; i0 += step) {
    uint32_t u[K], p[K], w[K], at[K];
#pragma unroll
    for (int q = 0; q < K; q++) {
      const int i = i0 + q * 256;
      u[q] = i < end ? __builtin_nontemporal_load(uid_sorted + i) : 0u;
      p[q] = i < end ? __builtin_nontemporal_load(pos + i) : 0u;  // the lookup's position: as is, or (bag, position inside it)
    }
#pragma unroll
    for (int q = 0; q < K; q++) {
      const int32_t lu = loc_u[u[q]];
      w[q] = lu >= 0 ? (uint32_t)lu : (kLocOverflow | (uint32_t)(-2 - lu));
      if (run_off[u[q] + 1] - run_off[u[q]] == 1) w[q] |= kLocSingle;
      at[q] = packed ? (uint32_t)offsets[p[q] >> within_bits] + (p[q] & within_mask) : p[q];
    }
#pragma unroll
    for (int q = 0; q < K; q++)
      if (i0 + q * 256 < end) loc[at[q]] = w[q];
  }
}

hipError_t launch_dedup_probe(const TableMeta *tm, const Geometry &g, const BatchBuf &b, SortScratch &ss,
                              const uint32_t *sorted_keys, const uint32_t *sorted_pos, int32_t *tags, int32_t *ts,
                              int32_t *freq, bool lfu, const Level2 &l2, int lock, hipStream_t s) {
  const int n = (int)b.n;
  if (n == 0) return hipSuccess;
  DedupOp d{tm, g.T, sorted_keys, sorted_pos, b.bag_of_pos, b.cnt, g.within_bits, b.d_offsets,
            b.maxp ? b.sorted_within : nullptr, b.uid_sorted, b.sorted_bag, b.uniq_key, b.run_off, b.uniq_sid,
            b.uniq_tab, nullptr};
  run_compaction(d, nullptr, n, n, ss.blk, b.cnt, s);
  SetHeadOp h{b.uniq_sid, b.run_off, b.touched};
  run_compaction(h, &b.cnt->n_uniq, 0, n, ss.blk, b.cnt, s);
  hipLaunchKernelGGL(worklist_count_kernel, dim3(kWorklistBlocks), dim3(256), 0, s, b.run_off, ss.wl, b.cnt);
  hipLaunchKernelGGL(worklist_emit_kernel, dim3(kWorklistBlocks), dim3(256), 0, s, b.run_off, b.uniq_tab, ss.wl, b.mid_idx,
                     b.heavy, b.heavy_sub, b.hg_count, b.cnt);
  if (!b.maxp) {  // the tile kernel's chunks and range starts (max pooling takes heavy rows a workgroup each)
    hipLaunchKernelGGL(heavy_group_kernel, dim3(1), dim3(256), 0, s, tm, g.T, b.hg_count, b.hg_count + g.T + 1, b.hchunks,
                       (long long)g.partial_slots, g.heavy_target, b.cnt);
    hipLaunchKernelGGL(heavy_order_kernel, dim3(g.T), dim3(64), 0, s, b.hg_count, b.hg_count + g.T + 1, b.heavy,
                       b.heavy_sub, b.run_off, b.hperm, b.cnt);
    hipLaunchKernelGGL(heavy_starts_kernel, dim3(256), dim3(256), 0, s, tm, b.batch, b.heavy, b.uniq_tab, b.run_off,
                       b.sorted_bag, b.hstart, b.cnt);
  }
  int64_t max_touched = (int64_t)g.total_sets + g.T;
  if (max_touched > n) max_touched = n;
  const int probe_blocks = (int)(max_touched < 65536 ? max_touched : 65536);
  auto probe = l2.on ? (lfu ? probe_kernel<true, true> : probe_kernel<false, true>)
                     : (lfu ? probe_kernel<true, false> : probe_kernel<false, false>);
  hipLaunchKernelGGL(probe, dim3(probe_blocks), dim3(kWave), 0, s, tm, g.T, g.ways, b.k, b.k - lock > 1 ? b.k - lock : 1, g.probe_min_windows, b.uniq_key, b.uniq_tab, b.touched,
                     tags, ts, freq, b.run_off, b.loc_u, b.status, b.old_tag, l2.tags2, l2.ts2, l2.factor,
                     l2.on ? b.src2 : nullptr, l2.on ? b.dst2 : nullptr, l2.on ? b.evict2 : nullptr, b.cnt);
  StatusOp st{tm, g.T, b.status, b.run_off, b.old_tag, b.uniq_key, b.uniq_tab, b.ins_idx, b.ins_tab, b.ins_slot,
              b.ins_old, b.ins_key, b.ins_src,
              b.byp_idx, b.byp_tab, b.byp_key, b.byp_src, b.loc_u,
              l2.on ? b.src2 : nullptr, l2.on ? b.dst2 : nullptr, l2.on ? b.evict2 : nullptr,
              l2.on ? b.ins_dst : nullptr, l2.on ? b.l2v_src : nullptr, l2.on ? b.l2v_dst : nullptr,
              l2.on ? b.l2v_key : nullptr, ss.tally, 0u, 0ull, nullptr};
  ss.tally_waves = run_compaction(st, &b.cnt->n_uniq, 0, n, ss.blk, b.cnt, s) * kScanWavesPerBlock;
  hipLaunchKernelGGL(finalize_kernel, dim3(TBE_FINALIZE_BLOCKS), dim3(256), 0, s, n, sorted_pos, b.uid_sorted, b.loc_u, b.run_off,
                     b.loc, b.d_offsets, g.within_bits, b.cnt);
  return hipGetLastError();
}

}  // namespace tbe
