// Data movement between the cache lines in HBM and the backing tier in pinned host memory
// (paper Section 5.5.3 data lookup/update, 5.5.4 data movement, one-level cache: missed rows
// are inserted from the lower tier, LRU rows are written back to it), arranged so that
// the host link works in both directions while the previous batch is still training
// (Section 5.7: prefetch ahead of training; Section 6.1: cache management overlapped with
// the computation of the batch before).
//
// For the batch being prefetched (k+1), with batch k possibly still training:
//   classify : a row wanted by k+1 whose backing-tier copy is being written in this very
//              window is "late".  A map over the sort keys says where its current value
//              is: in batch k's overflow copies (k bypassed it and trains on that copy)
//              or among the victims batch k parked (k evicted it).
//   transfer : victims of batch k, parked in the staging area when k was committed, go to
//              the backing tier; at the same time the rows batch k+1 inserts or bypasses
//              are fetched into HBM, except the late ones.  Runs on the link stream.
//   commit   : after batch k has trained: victims of k+1 move from their cache lines to
//              the staging area, the new rows move in; late rows are copied HBM to HBM from
//              where the map pointed.  Also writes batch k's overflow copies back.
// Host rows are reached through the pinned mapping, 16 lanes per row, 16 bytes per lane.
#include <hip/hip_fp16.h>
#include "tbe_internal.h"

namespace tbe {

typedef unsigned long long u64;
constexpr int kMoveLanes = 16;
constexpr int kLinkBlocks = 192;   // workgroups of the smaller kernels that write to the host link
constexpr int kLinkThreads = 1024;

// ---- deferred initialisation: counter-based normal numbers of (seed, table, row, element) ----
// z = centred sum of twelve 16-bit uniforms (three 64-bit hashes per element, the finaliser of
// splitmix64), integer arithmetic up to one fp32 product -- the stored bits are the same
// wherever the definition is evaluated.
__device__ inline u64 mix64(u64 x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

__device__ inline u64 init_table_key(u64 seed, int t) { return mix64(seed ^ ((u64)(t + 1) * 0xD1342543DE82EF95ull)); }

__device__ inline float init_value(u64 table_key, uint32_t row, uint32_t e, float scale) {
  int32_t s = -12 * 65536;
#pragma unroll
  for (int j = 0; j < 3; j++) {
    const u64 h = mix64(table_key + (u64)row * 0x2545F4914F6CDD1Dull + (u64)e * 3u + (u64)j);
    s += 2 * (int32_t)((h & 0xFFFFu) + ((h >> 16) & 0xFFFFu) + ((h >> 32) & 0xFFFFu) + (h >> 48)) + 4;
  }
  float v = __fmul_rn((float)s, scale);
  // The fp32 product is the value; the fp16 table stores its rounding.  Without this barrier the
  // compiler folds product and conversion into one mixed-precision instruction that rounds once,
  // which differs from rounding the fp32 value wherever that value is an fp16 tie.
  asm volatile("" : "+v"(v));
  return v;
}

// the 16 bytes of row `row` that start at element e0 (4 fp32 or 8 fp16 values), std * z each
__device__ inline uint4 init_chunk(u64 table_key, uint32_t row, int dtype, uint32_t e0, float std) {
  const float scale = std * 0x1p-17f;  // exact
  if (dtype == 0)
    return make_uint4(__float_as_uint(init_value(table_key, row, e0, scale)),
                      __float_as_uint(init_value(table_key, row, e0 + 1, scale)),
                      __float_as_uint(init_value(table_key, row, e0 + 2, scale)),
                      __float_as_uint(init_value(table_key, row, e0 + 3, scale)));
  uint32_t w[4];
  for (int i = 0; i < 4; i++)
    w[i] = (uint32_t)__half_as_ushort(__float2half_rn(init_value(table_key, row, e0 + 2 * i, scale))) |
           ((uint32_t)__half_as_ushort(__float2half_rn(init_value(table_key, row, e0 + 2 * i + 1, scale))) << 16);
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Has row `row` of table m a value yet?  If not, it gets one now: lane 0 of the group marks the
// row and tells the others what the mark was before.
__device__ inline bool needs_init(const TableMeta &m, uint32_t row, int lig) {
  const uint32_t bit = 1u << (row & 31);
  uint32_t before = 0;
  if (lig == 0) before = atomicOr(m.init_bits + (row >> 5), bit);
  before = __shfl(before, 0, kMoveLanes);
  return (before & bit) == 0;
}

typedef uint32_t mv_u32x4 __attribute__((ext_vector_type(4)));
// A row on its way to host memory: non-temporal stores (the transfer of the benchmark workload
// 5.52 -> 5.36 ms; non-temporal loads from host memory change nothing).
__device__ inline void copy_row_to_host(char *dst, const char *src, uint32_t bytes, int lig) {
  for (uint32_t c = lig * 16; c < bytes; c += kMoveLanes * 16) {
    const mv_u32x4 v = *(const mv_u32x4 *)(src + c);
    __builtin_nontemporal_store(v, (mv_u32x4 *)(dst + c));
  }
}
__device__ inline void copy_row(char *dst, const char *src, uint32_t bytes, int lig) {
  for (uint32_t c = lig * 16; c < bytes; c += kMoveLanes * 16) *(uint4 *)(dst + c) = *(const uint4 *)(src + c);
}

__global__ __launch_bounds__(kLinkThreads) void transfer_kernel(Staging st, const BatchCounters *cnt,
                                                       char *const *__restrict__ ins_src,
                                                       const int32_t *__restrict__ ins_tab,
                                                       const uint32_t *__restrict__ rb_of_table,
                                                       const uint32_t *__restrict__ ins_where,
                                                       char *const *__restrict__ byp_src,
                                                       const int32_t *__restrict__ byp_tab,
                                                       const uint32_t *__restrict__ byp_where, char *__restrict__ ovf,
                                                       char *const *__restrict__ l2v_src,
                                                       char *const *__restrict__ wb2_dst, char *out2_even,
                                                       char *out2_odd, int k, const TableMeta *__restrict__ di_tm,
                                                       u64 di_seed, float di_std,
                                                       const uint32_t *__restrict__ ins_key,
                                                       const uint32_t *__restrict__ byp_key, u64 *bytes_h2d,
                                                       u64 *bytes_d2h, const char *l2_lo, const char *l2_hi,
                                                       int pauses) {
  // Waves that wait on the host link slow the memory accesses of every wave that shares their CU,
  // so this kernel keeps its CUs to itself: a workgroup of 16 wavefronts that claims 128 vector
  // registers per lane fills the register files of a CU's four SIMDs, and no wave of another
  // kernel is placed beside it (the clobber makes the compiler allocate up to v127).
  asm volatile("" ::: "v127");
  const int bid = blockIdx.x, n_blocks = gridDim.x;
  const int n_wb = *st.wb_n;
  const int n_ins = (cnt && cnt->err == 0) ? cnt->n_ins : 0;
  const int n_byp = (cnt && cnt->err == 0) ? cnt->n_byp : 0;
  // One pass of the loop fetches item i and writes back slot i.  When there are more slots to write
  // than items to fetch (the overflow copies parked behind the victims), the surplus is paired with
  // the first passes (slot i + n) instead of forming a tail of passes that only write: the link's two
  // directions stay busy together to the end.
  const int n = max((n_wb + 1) / 2, max(n_ins, n_byp));
  const int group = (bid * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = n_blocks * blockDim.x / kMoveLanes;
  u64 in_b = 0, out_b = 0;
  const int wpar = st.wb_n[1] & 1;
  // emulated slower tier: rows of this pass that the group moved to or from the backing tier proper
  int slow_rows = 0;
  auto in_backing = [&](const char *p) { return pauses > 0 && !(p >= l2_lo && p < l2_hi); };
  auto write_back = [&](int w) {
    if (w >= n_wb) return;
    char *dst = st.wb_dst[w];
    uint8_t *skip = st.wb_skip[wpar] + w;
    if (*skip) {  // the batch being prefetched takes this row back from the parked copy: the
      dst = nullptr;  // line stays dirty in HBM and is written back when it is evicted again
      if (lig == 0) *skip = 0;
    }
    if (dst) {
      const uint32_t wrb = st.wb_rb[w];
      copy_row_to_host(dst, st.out[wpar] + (size_t)w * st.stride, wrb, lig);
      if (lig == 0) out_b += wrb;
      slow_rows += in_backing(dst);
    }
    if (wb2_dst) {  // second level: the row this victim pushed out of it goes to the lower tier
      char *dst2 = wb2_dst[w];
      uint8_t *skip2 = st.wb_skip[wpar] + st.max_inserts + w;
      if (dst2 && *skip2) {
        dst2 = nullptr;
        if (lig == 0) *skip2 = 0;
      }
      if (dst2) {
        const uint32_t wrb = st.wb_rb[w];
        copy_row_to_host(dst2, (wpar ? out2_odd : out2_even) + (size_t)w * st.stride, wrb, lig);
        if (lig == 0) out_b += wrb;
        slow_rows += in_backing(dst2);
      }
    }
  };
  for (int i = group; i < n; i += n_groups) {
    // issue the host read first, then the write-back, so both directions are busy
    uint4 fresh[4];
    uint32_t rb = 0;
    bool fetch = false, made_up = false;
    if (i < n_ins) {
      fetch = ins_where[i] == 0;
      if (fetch) {
        const int t = ins_tab[i];
        rb = rb_of_table[t];
        if (di_tm) {  // deferred initialisation: a row read for the first time gets its value here
          const TableMeta &m = di_tm[t];
          const uint32_t row = row_of_key(m, ins_key[i]);
          made_up = needs_init(m, row, lig);
          if (made_up) {
            const u64 tk = init_table_key(di_seed, t);
            const uint32_t esz = m.dtype == 0 ? 4u : 2u;
#pragma unroll
            for (int q = 0; q < 4; q++) {
              const uint32_t c = lig * 16 + q * kMoveLanes * 16;
              if (c < rb) fresh[q] = init_chunk(tk, row, m.dtype, c / esz, di_std);
            }
          }
        }
        if (!made_up) {
          const char *src = ins_src[i];
          slow_rows += in_backing(src);
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const uint32_t c = lig * 16 + q * kMoveLanes * 16;
            if (c < rb) fresh[q] = *(const uint4 *)(src + c);
          }
        }
      }
    }
    write_back(i);
    write_back(i + n);  // the slots beyond the loop's length ride along with the first ones
    if (l2v_src && i < n_ins) {  // second level: the row an insert's victim pushes out is read while its
      const char *src = l2v_src[i];  // line still holds it (the victim is written there by the next transfer)
      if (src) {
        const uint32_t vrb = rb_of_table[ins_tab[i]];
        copy_row(((k & 1) ? out2_odd : out2_even) + (size_t)i * st.stride, src, vrb, lig);
        if (lig == 0) in_b += vrb;
      }
    }
    if (fetch) {
      char *dst = st.in + (size_t)i * st.stride;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const uint32_t c = lig * 16 + q * kMoveLanes * 16;
        if (c < rb) *(uint4 *)(dst + c) = fresh[q];
      }
      if (lig == 0 && !made_up) in_b += rb;
    }
    if (i < n_byp && byp_where[i] == 0) {  // bypassed rows of this batch: HBM copy for its training
      const int t = byp_tab[i];
      const uint32_t brb = rb_of_table[t];
      bool fresh_row = false;
      if (di_tm) {
        const TableMeta &m = di_tm[t];
        const uint32_t row = row_of_key(m, byp_key[i]);
        fresh_row = needs_init(m, row, lig);
        if (fresh_row) {
          const u64 tk = init_table_key(di_seed, t);
          const uint32_t esz = m.dtype == 0 ? 4u : 2u;
          for (uint32_t c = lig * 16; c < brb; c += kMoveLanes * 16)
            *(uint4 *)(ovf + (size_t)i * st.stride + c) = init_chunk(tk, row, m.dtype, c / esz, di_std);
        }
      }
      if (!fresh_row) {
        copy_row(ovf + (size_t)i * st.stride, byp_src[i], brb, lig);
        if (lig == 0) in_b += brb;
        slow_rows += in_backing(byp_src[i]);
      }
    }
    if (pauses > 0) {  // the wavefront pauses once per backing-tier row its groups moved (a bounded delay: no wait on memory)
      int rows = 0;    // counted over the lanes still in the loop; a pass moves at most five rows per group
      for (int q = 1; q <= 5; q++) rows += __popcll(__ballot(lig == 0 && slow_rows >= q));
      for (int z = 0; z < rows * pauses; z++) __builtin_amdgcn_s_sleep(127);
      slow_rows = 0;
    }
  }
  for (int d = 32; d >= 1; d >>= 1) {
    in_b += __shfl_xor(in_b, d);
    out_b += __shfl_xor(out_b, d);
  }
  if ((threadIdx.x & 63) == 0) {
    if (in_b) atomicAdd(bytes_h2d, in_b);
    if (out_b) atomicAdd(bytes_d2h, out_b);
  }
}

__global__ void clear_wb_kernel(int32_t *wb_n) {
  if (threadIdx.x == 0) wb_n[0] = 0;
}

hipError_t launch_transfer(const BatchBuf *b, const Staging &st, const Level2 &l2, const DeferredInit &di,
                           const Throttle &th, int k, const uint32_t *rb_of_table, u64 *bytes_h2d, u64 *bytes_d2h,
                           hipStream_t s) {
  // How many waves wait on the host link, and where, decides how the link and the HBM-bound kernels
  // of the other streams slow each other.  Measured on the benchmark workload (step / transfer
  // kernel / prefetch stage / forward kernel while the transfer runs, ms; alone the forward takes
  // 0.20 and the prefetch stage 0.94):
  //   192 workgroups of 256 threads on two XCDs, CUs shared with other kernels : 6.40 / 5.63 / 4.8 / 0.45
  //   512 such workgroups on two XCDs (they fill them)                         : 6.92 / 5.42 / 5.8 / 0.23
  //   32 workgroups of 1024 threads, a CU each (any XCD)                       : 7.44 / 6.66 / 1.7 / 0.25
  //   48                                                                       : 6.31 / 5.55 / 1.9 / 0.28
  //   64                                                                       : 6.29 / 5.56 / 2.0 / 0.30
  //   96                                                                       : 6.60 / 5.84 / 3.1 / 0.42
  // (with the overflow copies riding along, later: 40 CUs 5.81 ms per step, 48: 5.67, 56: 5.70, 64: 5.93, 72: 6.03)
  // The link needs about 750 waves; given CUs of their own (48 of 256) they leave the other
  // streams' kernels at 1.3 to 2 times their stand-alone time instead of 2.5 to 5 times.
  hipLaunchKernelGGL(transfer_kernel, dim3(kLinkCus), dim3(kLinkThreads), 0, s, st, b ? b->cnt : nullptr,
                     b ? b->ins_src : nullptr, b ? b->ins_tab : nullptr, rb_of_table,
                     b ? b->ins_where : nullptr, b ? b->byp_src : nullptr, b ? b->byp_tab : nullptr,
                     b ? b->byp_where : nullptr, b ? b->ovf : nullptr, (b && l2.on) ? b->l2v_src : nullptr,
                     l2.on ? l2.wb2_dst : nullptr, l2.out2[0], l2.out2[1], k, b ? di.tm : nullptr, di.seed, di.std,
                     b ? b->ins_key : nullptr, b ? b->byp_key : nullptr, bytes_h2d, bytes_d2h, l2.lines_lo, l2.lines_hi,
                     th.pauses);
  hipLaunchKernelGGL(clear_wb_kernel, dim3(1), dim3(64), 0, s, st.wb_n);
  return hipGetLastError();
}

// Enter (set) or remove (clear) in the map the rows whose backing-tier copy batch `b` leaves
// stale for a while: the rows it evicted (parked victim i, written back by the next
// transfer) and the rows it bypassed (overflow copy j, written back after its backward).
// byp_mode: what the rows the batch bypassed get: kMarkClear, kMarkOverflow (overflow copy j of this
// batch) or kMarkParked (the next batch's commit parks copy j behind its own n_ins victims:
// kWhereParked | (next->n_ins + j)).  vic_mode: kMarkClear / kMarkOverflow (= set) for its victims, or
// kMarkKeep to leave them alone.
constexpr int kMarkClear = 0, kMarkOverflow = 1, kMarkParked = 2, kMarkKeep = 3;

__global__ __launch_bounds__(256) void mark_kernel(const TableMeta *__restrict__ tm, const BatchCounters *cnt,
                                                   const int32_t *__restrict__ ins_tab,
                                                   const int32_t *__restrict__ ins_old,
                                                   const uint32_t *__restrict__ byp_key,
                                                   char *const *__restrict__ l2v_src,
                                                   const uint32_t *__restrict__ l2v_key, uint32_t max_inserts,
                                                   uint32_t *where, int vic_mode, int byp_mode,
                                                   const BatchCounters *next_cnt, uint32_t overflow_code) {
  if (cnt->err) return;
  const int n_ins = vic_mode == kMarkKeep ? 0 : cnt->n_ins, n_byp = byp_mode == kMarkKeep ? 0 : cnt->n_byp;
  const int set = vic_mode != kMarkClear;
  const uint32_t park_base = (byp_mode == kMarkParked && next_cnt) ? (uint32_t)next_cnt->n_ins : 0u;
  const int stride = gridDim.x * blockDim.x;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_ins + n_byp; i += stride) {
    if (i < n_ins) {
      const int32_t old = ins_old[i];
      if (old >= 0) where[key_of_row(tm[ins_tab[i]], (uint32_t)old)] = set ? (kWhereParked | (uint32_t)i) : 0u;
      // the row pushed out of the second level is staged like a victim, behind the victims
      if (l2v_src && l2v_src[i]) where[l2v_key[i]] = set ? (kWhereParked | (max_inserts + (uint32_t)i)) : 0u;
    } else {
      const uint32_t j = (uint32_t)(i - n_ins);
      where[byp_key[j]] = byp_mode == kMarkOverflow ? (overflow_code | j) : byp_mode == kMarkParked ? (kWhereParked | (park_base + j)) : 0u;
    }
  }
}

__global__ __launch_bounds__(256) void classify_kernel(const BatchCounters *cnt, const uint32_t *__restrict__ ins_key,
                                                       const uint32_t *__restrict__ byp_key,
                                                       const uint32_t *__restrict__ where,
                                                       uint32_t *__restrict__ ins_where,
                                                       uint32_t *__restrict__ byp_where,
                                                       uint8_t *__restrict__ prev_wb_skip, u64 *n_late) {
  if (cnt->err) return;
  const int n_ins = cnt->n_ins, n_byp = cnt->n_byp;
  unsigned int late = 0;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_ins + n_byp; i += gridDim.x * blockDim.x) {
    const uint32_t code = where[i < n_ins ? ins_key[i] : byp_key[i - n_ins]];
    if (i < n_ins) ins_where[i] = code; else byp_where[i - n_ins] = code;
    // a victim the batch before parked and this batch wants back skips the trip to the host
    if (code & kWhereParked) prev_wb_skip[code & kWhereIndex] = 1;
    late += code != 0;
  }
  __shared__ unsigned int s_late[4];
  for (int d = 32; d >= 1; d >>= 1) late += __shfl_xor(late, d);
  if ((threadIdx.x & 63) == 0) s_late[threadIdx.x >> 6] = late;
  __syncthreads();
  if (threadIdx.x == 0) {
    late = s_late[0] + s_late[1] + s_late[2] + s_late[3];
    if (late) atomicAdd(n_late, (unsigned long long)late);
  }
}

hipError_t launch_classify_mark(const TableMeta *tm, const BatchBuf *pp, const BatchBuf *prev, const BatchBuf &cur,
                                const Staging &st, const Level2 &l2, u64 *n_late, hipStream_t s) {
  const uint32_t M = (uint32_t)st.max_inserts;
  hipLaunchKernelGGL(classify_kernel, dim3(512), dim3(256), 0, s, cur.cnt, cur.ins_key, cur.byp_key, st.where,
                     cur.ins_where, cur.byp_where, st.wb_skip[(cur.k - 1) & 1], n_late);
  // The marks move on in this order (a later one may overwrite an earlier one's entry, never the
  // other way round): the overflow copies that prev's commit parked are home once the transfer of
  // this batch is through; prev's victims likewise; prev's own overflow copies are either home
  // already or will be parked by this batch's commit behind its victims; then this batch's rows.
  if (pp)
    hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, pp->cnt, pp->ins_tab, pp->ins_old, pp->byp_key,
                       (char *const *)nullptr, (const uint32_t *)nullptr, M, st.where, kMarkKeep, kMarkClear,
                       (const BatchCounters *)nullptr, kWhereOverflow);
  if (prev)
    hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, prev->cnt, prev->ins_tab, prev->ins_old, prev->byp_key,
                       l2.on ? prev->l2v_src : nullptr, prev->l2v_key, M, st.where, kMarkClear,
                       cur.parks_prev ? kMarkParked : kMarkClear, cur.cnt, kWhereOverflow);
  hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, cur.cnt, cur.ins_tab, cur.ins_old, cur.byp_key,
                     l2.on ? cur.l2v_src : nullptr, cur.l2v_key, M, st.where, kMarkOverflow, kMarkOverflow,
                     (const BatchCounters *)nullptr, kWhereOverflow);
  return hipGetLastError();
}

// After a flush nothing is on its way to the backing tier any more: the marks of the last batch go,
// and those of the overflow copies its commit parked (parked_prev: the batch they belonged to).
hipError_t launch_unmark(const TableMeta *tm, const BatchBuf &last, const BatchBuf *parked_prev, const Staging &st,
                         const Level2 &l2, hipStream_t s) {
  if (parked_prev)
    hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, parked_prev->cnt, parked_prev->ins_tab,
                       parked_prev->ins_old, parked_prev->byp_key, (char *const *)nullptr, (const uint32_t *)nullptr,
                       (uint32_t)st.max_inserts, st.where, kMarkKeep, kMarkClear, (const BatchCounters *)nullptr, kWhereOverflow);
  hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, last.cnt, last.ins_tab, last.ins_old, last.byp_key,
                     l2.on ? last.l2v_src : nullptr, last.l2v_key, (uint32_t)st.max_inserts, st.where, kMarkClear, kMarkClear,
                     (const BatchCounters *)nullptr, kWhereOverflow);
  return hipGetLastError();
}

// ---- pipeline several batches deep ----
hipError_t launch_classify_mark_deep(const TableMeta *tm, const BatchBuf *prev, const BatchBuf &cur, int cur_buf,
                                     const Staging &st, u64 *n_late, hipStream_t s) {
  const uint32_t M = (uint32_t)st.max_inserts;
  hipLaunchKernelGGL(classify_kernel, dim3(512), dim3(256), 0, s, cur.cnt, cur.ins_key, cur.byp_key, st.where,
                     cur.ins_where, cur.byp_where, st.wb_skip[(cur.k - 1) & 1], n_late);
  if (prev)
    hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, prev->cnt, prev->ins_tab, prev->ins_old, prev->byp_key,
                       (char *const *)nullptr, (const uint32_t *)nullptr, M, st.where, kMarkClear, kMarkKeep,
                       (const BatchCounters *)nullptr, kWhereOverflow);
  hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, cur.cnt, cur.ins_tab, cur.ins_old, cur.byp_key,
                     (char *const *)nullptr, (const uint32_t *)nullptr, M, st.where, kMarkOverflow, kMarkOverflow,
                     (const BatchCounters *)nullptr, kWhereOverflow | ((uint32_t)cur_buf << kWhereBufShift));
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void unmark_bypassed_kernel(const BatchCounters *cnt, const uint32_t *__restrict__ byp_key,
                                                              uint32_t *where, uint32_t overflow_code) {
  if (cnt->err) return;
  const int n_byp = cnt->n_byp;
  for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < n_byp; j += gridDim.x * blockDim.x) {
    uint32_t *w = where + byp_key[j];
    if (*w == (overflow_code | (uint32_t)j)) *w = 0u;  // a later batch's entry for the same row stays
  }
}

hipError_t launch_unmark_bypassed(const BatchBuf &b, int buf, const Staging &st, hipStream_t s) {
  hipLaunchKernelGGL(unmark_bypassed_kernel, dim3(512), dim3(256), 0, s, b.cnt, b.byp_key, st.where,
                     kWhereOverflow | ((uint32_t)buf << kWhereBufShift));
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fixup_kernel(const TableMeta *__restrict__ tm, const BatchCounters *cnt,
                                                    const int32_t *__restrict__ ins_tab,
                                                    const uint32_t *__restrict__ ins_where,
                                                    const int32_t *__restrict__ ins_slot,
                                                    const uint32_t *__restrict__ ins_key,
                                                    const int32_t *__restrict__ byp_tab,
                                                    const uint32_t *__restrict__ byp_where, char *__restrict__ ovf,
                                                    OverflowCopies oc, uint32_t stride,
                                                    const uint32_t *__restrict__ rb_of_table, u64 *n_copied) {
  if (cnt->err) return;
  const int n_ins = cnt->n_ins, n_byp = cnt->n_byp;
  const int group = (blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = gridDim.x * blockDim.x / kMoveLanes;
  unsigned int copied = 0;
  for (int i = group; i < n_ins + n_byp; i += n_groups) {
    const bool ins = i < n_ins;
    const uint32_t code = ins ? ins_where[i] : byp_where[i - n_ins];
    if (!(code & kWhereOverflow)) continue;
    copied += lig == 0;
    const char *src = oc.of_buf[(code >> kWhereBufShift) & (kMaxBatchBufs - 1)] + (size_t)(code & kWhereBufIndex) * stride;
    if (ins) {
      const TableMeta &m = tm[ins_tab[i]];
      const int slot = ins_slot[i];
      copy_row(m.lines + (size_t)(slot - m.slot_base) * m.row_bytes, src, m.row_bytes, lig);
      // the row's accumulator was updated among those of all rows while it trained as a bypassed row
      if (lig == 0) m.slot_m[slot - m.slot_base] = m.dev_m[row_of_key(m, ins_key[i])];
    } else {
      const int j = i - n_ins;
      copy_row(ovf + (size_t)j * stride, src, rb_of_table[byp_tab[j]], lig);
    }
  }
  for (int d = 32; d >= 1; d >>= 1) copied += __shfl_xor(copied, d);
  if ((threadIdx.x & 63) == 0 && copied) atomicAdd(n_copied, (u64)copied);
}

hipError_t launch_fixup(const TableMeta *tm, const BatchBuf &b, const OverflowCopies &oc, const Staging &st,
                        const uint32_t *rb_of_table, u64 *n_copied, hipStream_t s) {
  if (b.n == 0) return hipSuccess;
  hipLaunchKernelGGL(fixup_kernel, dim3(1024), dim3(256), 0, s, tm, b.cnt, b.ins_tab, b.ins_where, b.ins_slot, b.ins_key,
                     b.byp_tab, b.byp_where, b.ovf, oc, st.stride, rb_of_table, n_copied);
  return hipGetLastError();
}

// The batch before (`prev`, may be absent) has trained when this runs, so a late row's
// current value is where its code says: prev's overflow copy or prev's parked victim, both
// still in HBM.  prev_mode says what becomes of prev's overflow rows: written back here (kPrevWrite), or
// parked behind this batch's victims for the next transfer to write them (kPrevPark): the link's
// write direction then carries them beside that transfer's fetches, which costs the transfer a
// hundredth of its time, instead of alone between two transfers.
template <bool DEEP>
__global__ __launch_bounds__(256) void commit_kernel(const TableMeta *__restrict__ tm, Staging st,
                                                     const BatchCounters *cnt, const int32_t *__restrict__ ins_tab,
                                                     const uint32_t *__restrict__ ins_where,
                                                     const int32_t *__restrict__ ins_slot,
                                                     const int32_t *__restrict__ ins_old,
                                                     const int32_t *__restrict__ byp_tab,
                                                     const uint32_t *__restrict__ byp_where, char *__restrict__ ovf,
                                                     const BatchCounters *prev_cnt,
                                                     char *const *__restrict__ prev_byp_src,
                                                     const int32_t *__restrict__ prev_byp_tab,
                                                     const char *__restrict__ prev_ovf, int wb_prev, int k,
                                                     char *const *__restrict__ ins_dst,
                                                     char *const *__restrict__ l2v_src,
                                                     char *const *__restrict__ l2v_dst, char **wb2_dst,
                                                     const char *__restrict__ out2_prev,
                                                     const uint32_t *__restrict__ rb_of_table,
                                                     const uint32_t *__restrict__ ins_key, u64 *bytes_d2h) {
  constexpr bool deep = DEEP;  // pipeline several batches deep (an instance of its own: the one-deep pipeline's commit
                               // is on the critical path of every step and keeps its code as it was)
  const uint32_t M = (uint32_t)st.max_inserts;  // map codes kWhereParked | (M + i): rows staged in out2
  const int n_prev = (prev_cnt && prev_cnt->err == 0) ? prev_cnt->n_byp : 0;
  const int group = (blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = gridDim.x * blockDim.x / kMoveLanes;
  if (cnt->err) {
    // This batch is refused (bad offsets or an index out of range) and does nothing, and no batch follows it
    // (the error sticks).  The batch before it has trained on its overflow copies, though: they go home now,
    // whatever was planned for them, so that a flush leaves the backing tier with that batch's updates.
    if (wb_prev != kPrevKeep) {
      u64 b = 0;
      for (int j = group; j < n_prev; j += n_groups) {
        const uint32_t rb = rb_of_table[prev_byp_tab[j]];
        copy_row_to_host(prev_byp_src[j], prev_ovf + (size_t)j * st.stride, rb, lig);
        if (lig == 0) b += rb;
      }
      for (int d = 32; d >= 1; d >>= 1) b += __shfl_xor(b, d);
      if ((threadIdx.x & 63) == 0 && b) atomicAdd(bytes_d2h, b);
    }
    return;
  }
  const int n_ins = cnt->n_ins, n_byp = cnt->n_byp;
  const int par = k & 1, ppar = par ^ 1;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st.wb_n[0] = n_ins + (wb_prev == kPrevPark ? n_prev : 0);
    st.wb_n[1] = par;
  }
  u64 out_b = 0;
  if (wb_prev == kPrevWrite)
    for (int j = group; j < n_prev; j += n_groups) {
      const uint32_t rb = rb_of_table[prev_byp_tab[j]];
      copy_row_to_host(prev_byp_src[j], prev_ovf + (size_t)j * st.stride, rb, lig);
      if (lig == 0) out_b += rb;
    }
  if (wb_prev == kPrevPark)
    for (int j = group; j < n_prev; j += n_groups) {
      const uint32_t rb = rb_of_table[prev_byp_tab[j]];
      const size_t slot = (size_t)n_ins + (size_t)j;
      copy_row(st.out[par] + slot * st.stride, prev_ovf + (size_t)j * st.stride, rb, lig);
      if (lig == 0) {
        st.wb_dst[slot] = prev_byp_src[j];
        st.wb_rb[slot] = rb;
      }
    }
  for (int i = group; i < n_ins; i += n_groups) {
    const TableMeta &m = tm[ins_tab[i]];
    const int slot = ins_slot[i];
    const int32_t old = ins_old[i];
    const uint32_t code = ins_where[i];
    const uint32_t rb = m.row_bytes;
    char *line = m.lines + (size_t)(slot - m.slot_base) * rb;
    const uint32_t ix = code & kWhereIndex;
    // (deep pipeline: an overflow copy may belong to a batch that has not trained yet -- the line gets the staging
    //  slot's content for now and the value, with its accumulator, before this batch's forward: fixup_kernel)
    const char *src = (code == 0 || (deep && (code & kWhereOverflow))) ? st.in + (size_t)i * st.stride
                      : (code & kWhereOverflow) ? prev_ovf + (size_t)ix * st.stride
                      : (out2_prev && ix >= M)  ? out2_prev + (size_t)(ix - M) * st.stride
                                                : st.out[ppar] + (size_t)ix * st.stride;
    char *park = st.out[par] + (size_t)i * st.stride;
    // The accumulators move with the rows: the victim's back among those of all rows, the new row's to the
    // slot (a row is in a cache line or among the others, never both, so the two differ).  Both are requested
    // before the row is copied, so that they travel beside it.
    float *sm = m.slot_m + (slot - m.slot_base);
    float m_victim = 0.f, m_fresh = 0.f;
    if (lig == 0) {
      m_victim = *sm;
      m_fresh = m.dev_m[row_of_key(m, ins_key[i])];
    }
    for (uint32_t c = lig * 16; c < rb; c += kMoveLanes * 16) {
      // The staged row and the parked victim pass through once: read and written around the caches, so that
      // the forward that follows does not start behind half a gigabyte of dirty lines (commit 0.274 -> 0.253 ms,
      // the forward after it 0.198 -> 0.186 ms).  The line itself is about to be read: it is stored as usual.
      const mv_u32x4 fresh = __builtin_nontemporal_load((const mv_u32x4 *)(src + c));
      if (old >= 0) __builtin_nontemporal_store(*(const mv_u32x4 *)(line + c), (mv_u32x4 *)(park + c));
      *(mv_u32x4 *)(line + c) = fresh;
    }
    if (lig == 0) {
      st.wb_dst[i] = old < 0 ? nullptr : ins_dst ? ins_dst[i] : m.host_w + (size_t)old * rb;
      st.wb_rb[i] = rb;
      if (wb2_dst) wb2_dst[i] = l2v_src[i] ? l2v_dst[i] : nullptr;
      if (old >= 0) m.dev_m[old] = m_victim;
      *sm = m_fresh;
    }
  }
  for (int j = group; j < n_byp; j += n_groups) {  // late bypassed rows
    const uint32_t code = byp_where[j];
    if (code == 0 || (deep && (code & kWhereOverflow))) continue;
    const uint32_t ix = code & kWhereIndex;
    const char *src = (code & kWhereOverflow) ? prev_ovf + (size_t)ix * st.stride
                      : (out2_prev && ix >= M) ? out2_prev + (size_t)(ix - M) * st.stride
                                              : st.out[ppar] + (size_t)ix * st.stride;
    copy_row(ovf + (size_t)j * st.stride, src, rb_of_table[byp_tab[j]], lig);
  }
  for (int d = 32; d >= 1; d >>= 1) out_b += __shfl_xor(out_b, d);
  if ((threadIdx.x & 63) == 0 && out_b) atomicAdd(bytes_d2h, out_b);
}

__global__ __launch_bounds__(256) void ovf_writeback_kernel(Staging st, const BatchCounters *cnt,
                                                            char *const *__restrict__ byp_src,
                                                            const int32_t *__restrict__ byp_tab,
                                                            const char *__restrict__ ovf,
                                                            const uint32_t *__restrict__ rb_of_table, u64 *bytes_d2h) {
  if (cnt->err) return;
  const int n_byp = cnt->n_byp;
  const int group = (blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = gridDim.x * blockDim.x / kMoveLanes;
  u64 out_b = 0;
  for (int j = group; j < n_byp; j += n_groups) {
    const uint32_t rb = rb_of_table[byp_tab[j]];
    copy_row_to_host(byp_src[j], ovf + (size_t)j * st.stride, rb, lig);
    if (lig == 0) out_b += rb;
  }
  for (int d = 32; d >= 1; d >>= 1) out_b += __shfl_xor(out_b, d);
  if ((threadIdx.x & 63) == 0 && out_b) atomicAdd(bytes_d2h, out_b);
}

// The overflow copies that batch b's commit parked behind its victims (those of the batch before
// it), written to the backing tier ahead of their turn: they must be home before b's own, newer
// copies of the same rows are written.  Their slots are emptied, so the next transfer passes them by.
__global__ __launch_bounds__(256) void parked_copies_writeback_kernel(Staging st, const BatchCounters *cnt,
                                                                      const BatchCounters *prev_cnt, u64 *bytes_d2h) {
  if (cnt->err || prev_cnt->err) return;
  const int base = cnt->n_ins, n = prev_cnt->n_byp;
  const char *out = st.out[st.wb_n[1] & 1];
  const int group = (blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = gridDim.x * blockDim.x / kMoveLanes;
  u64 out_b = 0;
  for (int j = group; j < n; j += n_groups) {
    const size_t slot = (size_t)base + (size_t)j;
    char *dst = st.wb_dst[slot];
    if (dst) {
      const uint32_t rb = st.wb_rb[slot];
      copy_row_to_host(dst, out + slot * st.stride, rb, lig);
      if (lig == 0) out_b += rb;
    }
  }
  __syncthreads();  // every lane of a group has read its slot's destination
  for (int j = group; j < n; j += n_groups)
    if (lig == 0) st.wb_dst[(size_t)base + (size_t)j] = nullptr;
  for (int d = 32; d >= 1; d >>= 1) out_b += __shfl_xor(out_b, d);
  if ((threadIdx.x & 63) == 0 && out_b) atomicAdd(bytes_d2h, out_b);
}

hipError_t launch_ovf_writeback(const BatchBuf &b, const BatchBuf *parked_prev, const Staging &st,
                                const uint32_t *rb_of_table, u64 *bytes_d2h, hipStream_t s) {
  if (parked_prev)
    hipLaunchKernelGGL(parked_copies_writeback_kernel, dim3(kLinkBlocks), dim3(256), 0, s, st, b.cnt, parked_prev->cnt,
                       bytes_d2h);
  if (b.n == 0) return hipGetLastError();
  hipLaunchKernelGGL(ovf_writeback_kernel, dim3(kLinkBlocks), dim3(256), 0, s, st, b.cnt, b.byp_src, b.byp_tab, b.ovf,
                     rb_of_table, bytes_d2h);
  return hipGetLastError();
}

hipError_t launch_commit(const TableMeta *tm, const BatchBuf &b, const BatchBuf *prev, int prev_mode, const Staging &st,
                         const Level2 &l2, const uint32_t *rb_of_table, u64 *bytes_d2h, bool deep, hipStream_t s) {
  auto kern = deep ? commit_kernel<true> : commit_kernel<false>;
  hipLaunchKernelGGL(kern, dim3(4096), dim3(256), 0, s, tm, st, b.cnt, b.ins_tab, b.ins_where, b.ins_slot,
                     b.ins_old, b.byp_tab, b.byp_where, b.ovf, prev ? prev->cnt : nullptr,
                     prev ? prev->byp_src : nullptr, prev ? prev->byp_tab : nullptr, prev ? prev->ovf : nullptr,
                     prev ? prev_mode : kPrevKeep, b.k, l2.on ? b.ins_dst : nullptr, l2.on ? b.l2v_src : nullptr,
                     l2.on ? b.l2v_dst : nullptr, l2.on ? l2.wb2_dst : nullptr, l2.out2[(b.k & 1) ^ 1], rb_of_table,
                     b.ins_key, bytes_d2h);
  return hipGetLastError();
}

// flush: every valid line goes to the backing tier, its accumulator to those of all rows (which the host code copies)
__global__ __launch_bounds__(256) void flush_kernel(const TableMeta *__restrict__ tm, int T, int64_t total_slots,
                                                    const int32_t *__restrict__ tags, u64 *bytes_d2h) {
  const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / kMoveLanes;
  u64 out_b = 0;
  for (int64_t slot = group; slot < total_slots; slot += n_groups) {
    const int32_t row = tags[slot];
    if (row < 0) continue;
    int lo = 0, hi = T - 1;  // table owning this slot: last t with slot_base <= slot
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((int64_t)tm[mid].slot_base <= slot) lo = mid; else hi = mid - 1;
    }
    const TableMeta &m = tm[lo];
    copy_row_to_host(m.host_w + (size_t)row * m.row_bytes, m.lines + (size_t)(slot - m.slot_base) * m.row_bytes, m.row_bytes, lig);
    if (lig == 0) {
      out_b += m.row_bytes;
      m.dev_m[row] = m.slot_m[slot - m.slot_base];  // the caller copies dev_m to the host; the line stays valid
    }
  }
  for (int d = 32; d >= 1; d >>= 1) out_b += __shfl_xor(out_b, d);
  if ((threadIdx.x & 63) == 0 && out_b) atomicAdd(bytes_d2h, out_b);
}

// flush of the second level: every valid line goes to its row in the lower tier (host to
// host through the GPU); the levels are exclusive, so no row is written twice
__global__ __launch_bounds__(256) void flush2_kernel(const TableMeta *__restrict__ tm, int T, int64_t total_slots2,
                                                     const int32_t *__restrict__ tags2, u64 *bytes_h2d,
                                                     u64 *bytes_d2h) {
  const int64_t group = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int64_t n_groups = (int64_t)gridDim.x * blockDim.x / kMoveLanes;
  u64 b = 0;
  for (int64_t slot = group; slot < total_slots2; slot += n_groups) {
    const int32_t row = tags2[slot];
    if (row < 0) continue;
    int lo = 0, hi = T - 1;  // table owning this slot: last t with slot2_base <= slot
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if ((int64_t)tm[mid].slot2_base <= slot) lo = mid; else hi = mid - 1;
    }
    const TableMeta &m = tm[lo];
    copy_row(m.host_w + (size_t)row * m.row_bytes, m.lines2 + (size_t)(slot - m.slot2_base) * m.row_bytes, m.row_bytes, lig);
    if (lig == 0) b += m.row_bytes;
  }
  for (int d = 32; d >= 1; d >>= 1) b += __shfl_xor(b, d);
  if ((threadIdx.x & 63) == 0 && b) {
    atomicAdd(bytes_h2d, b);
    atomicAdd(bytes_d2h, b);
  }
}

hipError_t launch_flush(const TableMeta *tm, const Geometry &g, const int32_t *tags, const Level2 &l2, u64 *bytes_h2d,
                        u64 *bytes_d2h, hipStream_t s) {
  if (g.total_slots)
    hipLaunchKernelGGL(flush_kernel, dim3(1024), dim3(256), 0, s, tm, g.T, g.total_slots, tags, bytes_d2h);
  if (l2.on && l2.total_slots2)
    hipLaunchKernelGGL(flush2_kernel, dim3(kLinkBlocks), dim3(256), 0, s, tm, g.T, l2.total_slots2, l2.tags2, bytes_h2d,
                       bytes_d2h);
  return hipGetLastError();
}

}  // namespace tbe
