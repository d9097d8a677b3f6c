// Index dedup, part 1: sort keys for every lookup of a batch and a stable LSD radix sort
// of (key, position) pairs.  The paper does not describe this step; it serves the
// "group the indices" part of the tag/state lookup (Section 5.5.1) on a 64-wide machine.
#include "tbe_internal.h"

namespace tbe {

// --------------------------------------------------------------------------------------
// key generation: 8 lanes per bag, 64-byte coalesced reads of the bag's indices
// --------------------------------------------------------------------------------------
constexpr int kKeygenLanes = 8;

// Does every bag fit the packed payload?  (cnt->packed starts at 1.)
__global__ __launch_bounds__(256) void baglen_kernel(int64_t nb, const int64_t *__restrict__ offsets, int within_bits,
                                                     BatchCounters *cnt) {
  const int64_t bag = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool too_long = bag < nb && offsets[bag + 1] - offsets[bag] > (1ll << within_bits);
  if (__ballot(too_long) && (threadIdx.x & 63) == 0) atomicMin(&cnt->packed, 0);
}

__global__ __launch_bounds__(256) void keygen_kernel(const TableMeta *__restrict__ tm, int T, int B, int64_t N,
                                                     const int64_t *__restrict__ indices,
                                                     const int64_t *__restrict__ offsets, uint32_t *__restrict__ keys,
                                                     uint32_t *__restrict__ vals, int32_t *__restrict__ bag_of_pos,
                                                     float *__restrict__ inv_len, int within_bits,
                                                     BatchCounters *cnt) {
  const int64_t nb = (int64_t)T * B;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t bag = gid / kKeygenLanes;
  const int sub = (int)(gid % kKeygenLanes);
  if (bag >= nb) return;
  int64_t lo = offsets[bag], hi = offsets[bag + 1];
  bool bad = lo < 0 || hi > N || lo > hi;
  if (bag == 0 && lo != 0) bad = true;
  if (bag == nb - 1 && hi != N) bad = true;
  if (bad) {
    if (sub == 0) atomicMax(&cnt->err, 1 /* -TBE_EINVAL */);
    return;
  }
  // mean pooling (Section 2.1.1): a lookup of a bag of L lookups weighs 1/L
  if (inv_len && sub == 0) inv_len[bag] = hi > lo ? 1.0f / (float)(hi - lo) : 0.0f;
  const int t = (int)(bag / B);
  const TableMeta m = tm[t];
  const bool packed = cnt->packed != 0;
  // two indices per lane and step, both requested before either is used (the loop is bound by the latency
  // of these reads: a bag has a few dozen lookups, so a lane makes only a few steps)
  auto emit = [&](int64_t j, int64_t r) {
    if (r < 0 || r >= m.rows) {
      atomicMax(&cnt->err, 2 /* -TBE_ERANGE */);
      r = 0;
    }
    keys[j] = key_of_row(m, (uint32_t)r);
    if (packed) {
      vals[j] = ((uint32_t)bag << within_bits) | (uint32_t)(j - lo);
    } else {
      vals[j] = (uint32_t)j;
      bag_of_pos[j] = (int32_t)bag;
    }
  };
  for (int64_t j = lo + sub; j < hi; j += 2 * kKeygenLanes) {
    const bool second = j + kKeygenLanes < hi;
    const int64_t r0 = indices[j];
    const int64_t r1 = second ? indices[j + kKeygenLanes] : 0;
    emit(j, r0);
    if (second) emit(j + kKeygenLanes, r1);
  }
}

__global__ void reset_counters_kernel(BatchCounters *cnt, int within_bits, int32_t *heavy_per_table, int T) {
  for (int t = threadIdx.x; t < T; t += blockDim.x) heavy_per_table[t] = 0;
  if (threadIdx.x == 0) {
    cnt->n_uniq = cnt->n_touched = cnt->n_ins = cnt->n_byp = cnt->n_heavy = cnt->err = 0;
    cnt->n_mid = cnt->n_hchunks = 0;
    cnt->h_ranges = 1;
    cnt->hits = cnt->evictions = cnt->hit_lookups = 0;
    cnt->l2_hits = cnt->l2_demotions = cnt->l2_evictions = cnt->l2_bypasses = 0;
    cnt->packed = within_bits > 0 ? 1 : 0;
  }
}

hipError_t launch_keygen(const TableMeta *tm, const Geometry &g, const BatchBuf &b, uint32_t *keys, uint32_t *vals,
                         hipStream_t s) {
  hipLaunchKernelGGL(reset_counters_kernel, dim3(1), dim3(64), 0, s, b.cnt, g.within_bits, b.hg_count, g.T);
  const int64_t nb = (int64_t)g.T * b.batch;
  if (g.within_bits > 0 && nb > 0)
    hipLaunchKernelGGL(baglen_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, s, nb, b.d_offsets, g.within_bits,
                       b.cnt);
  const int64_t threads = (int64_t)g.T * b.batch * kKeygenLanes;
  if (threads > 0) {
    const int64_t blocks = (threads + 255) / 256;
    hipLaunchKernelGGL(keygen_kernel, dim3((unsigned)blocks), dim3(256), 0, s, tm, g.T, b.batch, b.n, b.d_indices,
                       b.d_offsets, keys, vals, b.bag_of_pos, b.mean ? b.inv_len : nullptr, g.within_bits, b.cnt);
  }
  return hipGetLastError();
}

// --------------------------------------------------------------------------------------
// LSD radix sort, digits of up to 8 bits (9 where that saves a pass), three kernels per pass:
//   upsweep   : per-block digit histogram of the block's contiguous chunk
//   scan      : per digit, exclusive scan of its counts over the blocks, and digit totals
//   downsweep : the block walks its chunk tile by tile; inside a tile every wave ranks
//               its keys with ballot matching (stable), the tile is ordered by digit in
//               LDS and written out so that neighbouring lanes hit neighbouring addresses
// --------------------------------------------------------------------------------------
constexpr int kSortTile = 4096;        // keys of a tile
constexpr int kMaxRadix = 512;         // a pass sorts by a digit of up to 9 bits; one thread per digit value
constexpr int kMaxSortBlocks = 1024;
constexpr int kUpsweepKeys = 4;  // keys a thread of the counting pass has in flight (8 and 16: no faster)

template <int RB>
__global__ __launch_bounds__(1 << RB) void sort_upsweep_kernel(const uint32_t *__restrict__ keys, int n, int shift,
                                                               uint32_t mask, int chunk, uint32_t *__restrict__ hist) {
  constexpr int kRadix = 1 << RB, kSortThreads = kRadix;
  __shared__ uint32_t h[kRadix];
  const int tid = threadIdx.x;
  h[tid] = 0;
  __syncthreads();
  const int base = blockIdx.x * chunk;
  const int end = min(n, base + chunk);
  // Several keys per thread and step, their loads in flight together.  After the first pass equal keys lie side
  // by side, and a power-law batch has keys with thousands of copies: a wavefront whose 64 keys share one digit
  // adds them with one atomic instead of 64 to the same LDS word.
  for (int i0 = base; i0 < end; i0 += kUpsweepKeys * kSortThreads) {
    uint32_t k[kUpsweepKeys];
#pragma unroll
    for (int q = 0; q < kUpsweepKeys; q++) {
      const int i = i0 + q * kSortThreads + tid;
      k[q] = i < end ? keys[i] : 0u;
    }
#pragma unroll
    for (int q = 0; q < kUpsweepKeys; q++) {
      const bool valid = i0 + q * kSortThreads + tid < end;
      const uint32_t d = valid ? (k[q] >> shift) & mask : 0xFFFFFFFFu;
      const uint32_t d0 = __shfl(d, 0, 64);
      if (__all(d == d0)) {
        if ((tid & 63) == 0 && valid) atomicAdd(&h[d0], 64u);
      } else if (valid) {
        atomicAdd(&h[d], 1u);
      }
    }
  }
  __syncthreads();
  hist[tid * gridDim.x + blockIdx.x] = h[tid];
}

// One block per digit: exclusive scan, over the sort blocks, of that digit's counts (in
// place) and the digit's total.  nb <= kMaxSortBlocks.
__global__ __launch_bounds__(256) void sort_scan_kernel(uint32_t *hist, int nb, uint32_t *digit_total) {
  // 256 threads with four counts each (not one thread per count): a workgroup of 1024 threads waits for
  // half a CU's wave slots at once, which took this small kernel 60 to 80 us instead of 5 whenever the
  // other streams' kernels kept the CUs busy
  constexpr int kPer = kMaxSortBlocks / 256;
  __shared__ uint32_t wsum[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t *row = hist + (size_t)blockIdx.x * nb;
  uint32_t v[kPer], mine = 0;
#pragma unroll
  for (int q = 0; q < kPer; q++) {
    const int i = tid * kPer + q;
    v[q] = i < nb ? row[i] : 0u;
    mine += v[q];
  }
  uint32_t incl = mine;
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t o = __shfl_up(incl, d);
    if (lane >= d) incl += o;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  uint32_t wb = 0;
  for (int w = 0; w < wave; w++) wb += wsum[w];
  uint32_t pre = wb + incl - mine;
#pragma unroll
  for (int q = 0; q < kPer; q++) {
    const int i = tid * kPer + q;
    if (i < nb) row[i] = pre;
    pre += v[q];
  }
  if (tid == 255) digit_total[blockIdx.x] = wb + incl;
}

template <int RB>
__global__ __launch_bounds__(1 << RB) void sort_downsweep_kernel(
    const uint32_t *__restrict__ keys_in, const uint32_t *__restrict__ vals_in, uint32_t *__restrict__ keys_out,
    uint32_t *__restrict__ vals_out, int n, int shift, uint32_t mask, int chunk, const uint32_t *__restrict__ hist,
    const uint32_t *__restrict__ digit_total) {
  constexpr int kRadix = 1 << RB, kSortThreads = kRadix, kWaves = kSortThreads / kWave;
  // keys per thread and tile; the 9-bit pass with 4, 6, 12, 16 keys per thread: 77, 69, 68, 71 us against 62
  constexpr int kSortItems = RB == 9 ? 8 : 16;
  constexpr int kTile = kSortThreads * kSortItems;  // 4096 either way; a block's chunk is a multiple of it
  __shared__ uint32_t s_keys[kTile];
  __shared__ uint32_t s_vals[kTile];
  __shared__ uint32_t s_cnt[kWaves][kRadix];  // per wave and digit: count, later exclusive prefix over waves
  __shared__ uint32_t s_dstart[kRadix];       // first tile-sorted position of each digit
  __shared__ uint32_t s_gbase[kRadix];        // next global output position of each digit for this block
  __shared__ uint32_t s_wtot[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const int block_base = blockIdx.x * chunk;
  const int block_end = min(n, block_base + chunk);
  {  // first output position of digit tid for this block: digits before it + blocks before this one
    const uint32_t tot = digit_total[tid];
    uint32_t incl = tot;
    for (int dd = 1; dd < 64; dd <<= 1) {
      uint32_t o = __shfl_up(incl, dd);
      if (lane >= dd) incl += o;
    }
    if (lane == 63) s_wtot[wave] = incl;
    __syncthreads();
    uint32_t wb = 0;
    for (int w = 0; w < wave; w++) wb += s_wtot[w];
    s_gbase[tid] = wb + incl - tot + hist[tid * gridDim.x + blockIdx.x];
    __syncthreads();
  }

  for (int tile = block_base; tile < block_end; tile += kTile) {
    for (int w = 0; w < kWaves; w++) s_cnt[w][tid] = 0;
    __syncthreads();
    uint32_t key[kSortItems], val[kSortItems], rank[kSortItems];
    const int seg = tile + wave * (kWave * kSortItems);
#pragma unroll
    for (int q = 0; q < kSortItems; q++) {
      const int i = seg + q * kWave + lane;
      const bool valid = i < block_end;
      key[q] = valid ? keys_in[i] : 0xFFFFFFFFu;
      val[q] = valid ? vals_in[i] : 0u;
    }
#pragma unroll
    for (int q = 0; q < kSortItems; q++) {
      const int i = seg + q * kWave + lane;
      const bool valid = i < block_end;
      const uint32_t d = (key[q] >> shift) & mask;
      uint64_t peers = __ballot(valid);
#pragma unroll
      for (int bit = 0; bit < RB; bit++) {
        const bool on = (d >> bit) & 1u;
        const uint64_t bal = __ballot(on);
        peers &= on ? bal : ~bal;
      }
      const uint32_t below = __popcll(peers & lt_mask);
      uint32_t prev = 0;
      if (valid && below == 0) prev = atomicAdd(&s_cnt[wave][d], (uint32_t)__popcll(peers));
      const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : lane;
      prev = __shfl(prev, leader);
      rank[q] = prev + below;
    }
    __syncthreads();
    // thread tid owns digit tid: totals, prefix over waves, start of the digit in the tile
    uint32_t total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; w++) {
      const uint32_t c = s_cnt[w][tid];
      s_cnt[w][tid] = total;
      total += c;
    }
    uint32_t incl = total;
    for (int dd = 1; dd < 64; dd <<= 1) {
      uint32_t o = __shfl_up(incl, dd);
      if (lane >= dd) incl += o;
    }
    if (lane == 63) s_wtot[wave] = incl;
    __syncthreads();
    uint32_t wb = 0;
    for (int w = 0; w < wave; w++) wb += s_wtot[w];
    const uint32_t dstart = wb + incl - total;
    s_dstart[tid] = dstart;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kSortItems; q++) {
      const int i = seg + q * kWave + lane;
      if (i < block_end) {
        const uint32_t d = (key[q] >> shift) & mask;
        const uint32_t p = s_dstart[d] + s_cnt[wave][d] + rank[q];
        s_keys[p] = key[q];
        s_vals[p] = val[q];
      }
    }
    __syncthreads();
    const int tile_n = min(kTile, block_end - tile);
    for (int p = tid; p < tile_n; p += kSortThreads) {
      const uint32_t k = s_keys[p];
      const uint32_t d = (k >> shift) & mask;
      const uint32_t gpos = s_gbase[d] + ((uint32_t)p - s_dstart[d]);
      keys_out[gpos] = k;
      vals_out[gpos] = s_vals[p];
    }
    __syncthreads();
    s_gbase[tid] += total;
    __syncthreads();
  }
}

// Sorts ss.keys[0]/vals[0] (n pairs) by the low g.key_bits bits; *result_buf tells which of
// the two buffers holds the result.
hipError_t launch_sort(const Geometry &g, SortScratch &ss, int64_t n, int *result_buf, hipStream_t s) {
  *result_buf = 0;
  if (n <= 1) return hipSuccess;
  // 8-bit digits, except that keys of 25 to 27 bits (32 tables of a million rows make 25) take three passes, some of
  // them by a 9-bit digit, instead of four
  const int passes = (g.key_bits >= 25 && g.key_bits <= 27) ? 3 : (g.key_bits + 7) / 8;
  const int64_t tiles = (n + kSortTile - 1) / kSortTile;
  const int blocks = (int)(tiles < kMaxSortBlocks ? tiles : kMaxSortBlocks);
  const int64_t tiles_per_block = (tiles + blocks - 1) / blocks;
  const int chunk = (int)(tiles_per_block * kSortTile);
  const int used_blocks = (int)((n + chunk - 1) / chunk);
  int cur = 0, shift = 0;
  uint32_t *digit_total = ss.hist + kMaxRadix * kMaxSortBlocks;
  for (int p = 0; p < passes; p++) {
    const int left = g.key_bits - shift;
    const int w = (left + (passes - p) - 1) / (passes - p);  // balanced digit widths, the wider ones first
    const uint32_t mask = (1u << w) - 1u;
    if (w > 8) {
      hipLaunchKernelGGL(sort_upsweep_kernel<9>, dim3(used_blocks), dim3(512), 0, s, ss.keys[cur], (int)n, shift, mask,
                         chunk, ss.hist);
      hipLaunchKernelGGL(sort_scan_kernel, dim3(512), dim3(256), 0, s, ss.hist, used_blocks, digit_total);
      hipLaunchKernelGGL(sort_downsweep_kernel<9>, dim3(used_blocks), dim3(512), 0, s, ss.keys[cur], ss.vals[cur],
                         ss.keys[cur ^ 1], ss.vals[cur ^ 1], (int)n, shift, mask, chunk, ss.hist, digit_total);
    } else {
      hipLaunchKernelGGL(sort_upsweep_kernel<8>, dim3(used_blocks), dim3(256), 0, s, ss.keys[cur], (int)n, shift, mask,
                         chunk, ss.hist);
      hipLaunchKernelGGL(sort_scan_kernel, dim3(256), dim3(256), 0, s, ss.hist, used_blocks, digit_total);
      hipLaunchKernelGGL(sort_downsweep_kernel<8>, dim3(used_blocks), dim3(256), 0, s, ss.keys[cur], ss.vals[cur],
                         ss.keys[cur ^ 1], ss.vals[cur ^ 1], (int)n, shift, mask, chunk, ss.hist, digit_total);
    }
    shift += w;
    cur ^= 1;
  }
  *result_buf = cur;
  return hipGetLastError();
}

}  // namespace tbe
