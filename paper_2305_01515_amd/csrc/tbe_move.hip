// Data movement between the cache lines in HBM and the backing tier in pinned host memory
// (paper Section 5.5.3 data lookup/update, 5.5.4 data movement, one-level cache: missed rows
// are inserted from the lower tier, LRU rows are written back to it), arranged so that
// the host link works in both directions while the previous batch is still training
// (Section 5.7: prefetch ahead of training; Section 6.1: cache management overlapped with
// the computation of the batch before).
//
// For the batch being prefetched (k+1), with batch k possibly still training:
//   classify : a row to insert whose backing-tier copy is being written in this very
//              window (evicted by k, or bypassed by k and updated in place by k's
//              backward; both are marked in a bitmap over the sort keys) is flagged late.
//   transfer : victims of batch k, parked in the staging area when k was committed, go to
//              the backing tier; at the same time the rows batch k+1 inserts are fetched
//              into the staging area, except the late ones.  Runs on the link stream.
//   commit   : after batch k has trained: victims of k+1 move from their cache lines to
//              the staging area, the new rows move in (late rows straight from the host).
// Host rows are reached through the pinned mapping, 16 lanes per row, 16 bytes per lane.
#include "tbe_internal.h"

namespace tbe {

typedef unsigned long long u64;
constexpr int kMoveLanes = 16;
constexpr int kLinkBlocks = 128;

__device__ inline void copy_row(char *dst, const char *src, uint32_t bytes, int lig) {
  for (uint32_t c = lig * 16; c < bytes; c += kMoveLanes * 16) *(uint4 *)(dst + c) = *(const uint4 *)(src + c);
}

__global__ __launch_bounds__(256) void transfer_kernel(Staging st, const BatchCounters *cnt,
                                                       char *const *__restrict__ ins_src,
                                                       const int32_t *__restrict__ ins_tab,
                                                       const uint32_t *__restrict__ rb_of_table,
                                                       const uint8_t *__restrict__ ins_late,
                                                       char *const *__restrict__ byp_src,
                                                       const int32_t *__restrict__ byp_tab,
                                                       const uint8_t *__restrict__ byp_late, char *__restrict__ ovf,
                                                       u64 *bytes_h2d, u64 *bytes_d2h) {
  const int n_wb = *st.wb_n;
  const int n_ins = (cnt && cnt->err == 0) ? cnt->n_ins : 0;
  const int n_byp = (cnt && cnt->err == 0) ? cnt->n_byp : 0;
  const int n = max(n_wb, max(n_ins, n_byp));
  const int group = (blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = gridDim.x * blockDim.x / kMoveLanes;
  u64 in_b = 0, out_b = 0;
  for (int i = group; i < n; i += n_groups) {
    // issue the host read first, then the write-back, so both directions are busy
    uint4 fresh[4];
    uint32_t rb = 0;
    bool fetch = false;
    if (i < n_ins) {
      fetch = ins_late[i] == 0;
      if (fetch) {
        rb = rb_of_table[ins_tab[i]];
        const char *src = ins_src[i];
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const uint32_t c = lig * 16 + q * kMoveLanes * 16;
          if (c < rb) fresh[q] = *(const uint4 *)(src + c);
        }
      }
    }
    if (i < n_wb) {
      char *dst = st.wb_dst[i];
      if (dst) {
        const uint32_t wrb = st.wb_rb[i];
        copy_row(dst, st.out + (size_t)i * st.stride, wrb, lig);
        if (lig == 0) out_b += wrb;
      }
    }
    if (fetch) {
      char *dst = st.in + (size_t)i * st.stride;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const uint32_t c = lig * 16 + q * kMoveLanes * 16;
        if (c < rb) *(uint4 *)(dst + c) = fresh[q];
      }
      if (lig == 0) in_b += rb;
    }
    if (i < n_byp && byp_late[i] == 0) {  // bypassed rows of this batch: HBM copy for its training
      const uint32_t brb = rb_of_table[byp_tab[i]];
      copy_row(ovf + (size_t)i * st.stride, byp_src[i], brb, lig);
      if (lig == 0) in_b += brb;
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
  if (threadIdx.x == 0) *wb_n = 0;
}

hipError_t launch_transfer(const BatchBuf *b, const Staging &st, const uint32_t *rb_of_table, u64 *bytes_h2d,
                           u64 *bytes_d2h, hipStream_t s) {
  // 128 workgroups keep the link at its two-way peak; more of them only add host requests in
  // flight, which slows HBM-bound kernels on the other streams (measured: 256 blocks halve a
  // concurrent copy kernel's bandwidth, 64 blocks cost it 20 % but lose 5 % of the link)
  hipLaunchKernelGGL(transfer_kernel, dim3(kLinkBlocks), dim3(256), 0, s, st, b ? b->cnt : nullptr,
                     b ? b->ins_src : nullptr, b ? b->ins_tab : nullptr, rb_of_table,
                     b ? b->ins_late : nullptr, b ? b->byp_src : nullptr, b ? b->byp_tab : nullptr,
                     b ? b->byp_late : nullptr, b ? b->ovf : nullptr, bytes_h2d, bytes_d2h);
  hipLaunchKernelGGL(clear_wb_kernel, dim3(1), dim3(64), 0, s, st.wb_n);
  return hipGetLastError();
}

// set or clear, in the dirty bitmap, the rows whose backing-tier copy batch `b` writes:
// the rows it evicted (written back by the next transfer) and the rows it bypassed
// (updated in place by its backward)
__global__ __launch_bounds__(256) void mark_kernel(const TableMeta *__restrict__ tm, const BatchCounters *cnt,
                                                   const int32_t *__restrict__ ins_idx,
                                                   const int32_t *__restrict__ ins_tab,
                                                   const int32_t *__restrict__ old_tag,
                                                   const int32_t *__restrict__ byp_idx,
                                                   const uint32_t *__restrict__ uniq_key, uint32_t *dirty, int set) {
  if (cnt->err) return;
  const int n_ins = cnt->n_ins, n_byp = cnt->n_byp;
  const int stride = gridDim.x * blockDim.x;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_ins + n_byp; i += stride) {
    uint32_t key;
    if (i < n_ins) {
      const int32_t old = old_tag[ins_idx[i]];
      if (old < 0) continue;
      key = key_of_row(tm[ins_tab[i]], (uint32_t)old);
    } else {
      key = uniq_key[byp_idx[i - n_ins]];
    }
    if (set) atomicOr(&dirty[key >> 5], 1u << (key & 31));
    else atomicAnd(&dirty[key >> 5], ~(1u << (key & 31)));
  }
}

__global__ __launch_bounds__(256) void classify_kernel(const BatchCounters *cnt, const uint32_t *__restrict__ ins_key,
                                                       const uint32_t *__restrict__ byp_key,
                                                       const uint32_t *__restrict__ dirty,
                                                       uint8_t *__restrict__ ins_late, uint8_t *__restrict__ byp_late,
                                                       u64 *n_late) {
  if (cnt->err) return;
  const int n_ins = cnt->n_ins, n_byp = cnt->n_byp;
  unsigned int late = 0;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_ins + n_byp; i += gridDim.x * blockDim.x) {
    const uint32_t key = i < n_ins ? ins_key[i] : byp_key[i - n_ins];
    const uint32_t bit = (dirty[key >> 5] >> (key & 31)) & 1u;
    if (i < n_ins) ins_late[i] = (uint8_t)bit; else byp_late[i - n_ins] = (uint8_t)bit;
    late += bit;
  }
  for (int d = 32; d >= 1; d >>= 1) late += __shfl_xor(late, d);
  if ((threadIdx.x & 63) == 0 && late) atomicAdd(n_late, (unsigned long long)late);
}

hipError_t launch_classify_mark(const TableMeta *tm, const BatchBuf *prev, const BatchBuf &cur, const Staging &st,
                                u64 *n_late, hipStream_t s) {
  hipLaunchKernelGGL(classify_kernel, dim3(512), dim3(256), 0, s, cur.cnt, cur.ins_key, cur.byp_key, st.dirty, cur.ins_late,
                     cur.byp_late, n_late);
  if (prev)
    hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, prev->cnt, prev->ins_idx, prev->ins_tab, prev->old_tag,
                       prev->byp_idx, prev->uniq_key, st.dirty, 0);
  hipLaunchKernelGGL(mark_kernel, dim3(512), dim3(256), 0, s, tm, cur.cnt, cur.ins_idx, cur.ins_tab, cur.old_tag,
                     cur.byp_idx, cur.uniq_key, st.dirty, 1);
  return hipGetLastError();
}

// j with keys[j] == key in the ascending array keys[0..n), or -1
__device__ inline int find_key(const uint32_t *keys, int n, uint32_t key) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (keys[mid] < key) lo = mid + 1; else hi = mid;
  }
  return (lo < n && keys[lo] == key) ? lo : -1;
}

// The batch before (`prev`, may be absent) has trained when this runs.  A late row was
// either bypassed by prev -- then its current value is prev's overflow copy, still in HBM
// -- or evicted by prev -- then the backing tier is current by now.  With wb_prev set the
// kernel also writes prev's overflow rows back, so the link carries both directions.
__global__ __launch_bounds__(256) void commit_kernel(const TableMeta *__restrict__ tm, Staging st,
                                                     const BatchCounters *cnt, const int32_t *__restrict__ ins_idx,
                                                     const int32_t *__restrict__ ins_tab,
                                                     const uint32_t *__restrict__ ins_key,
                                                     char *const *__restrict__ ins_src,
                                                     const uint8_t *__restrict__ ins_late,
                                                     const int32_t *__restrict__ loc_u,
                                                     const int32_t *__restrict__ old_tag,
                                                     char *const *__restrict__ byp_src,
                                                     const int32_t *__restrict__ byp_tab,
                                                     const uint32_t *__restrict__ byp_key,
                                                     const uint8_t *__restrict__ byp_late, char *__restrict__ ovf,
                                                     const BatchCounters *prev_cnt,
                                                     const uint32_t *__restrict__ prev_byp_key,
                                                     char *const *__restrict__ prev_byp_src,
                                                     const int32_t *__restrict__ prev_byp_tab,
                                                     const char *__restrict__ prev_ovf, int wb_prev,
                                                     const uint32_t *__restrict__ rb_of_table, u64 *bytes_h2d,
                                                     u64 *bytes_d2h) {
  if (cnt->err) return;
  const int n_ins = cnt->n_ins, n_byp = cnt->n_byp;
  const int n_prev = (prev_cnt && prev_cnt->err == 0) ? prev_cnt->n_byp : 0;
  const int group = (blockIdx.x * blockDim.x + threadIdx.x) / kMoveLanes;
  const int lig = threadIdx.x % kMoveLanes;
  const int n_groups = gridDim.x * blockDim.x / kMoveLanes;
  if (blockIdx.x == 0 && threadIdx.x == 0) *st.wb_n = n_ins;
  u64 in_b = 0, out_b = 0;
  if (wb_prev)
    for (int j = group; j < n_prev; j += n_groups) {
      const uint32_t rb = rb_of_table[prev_byp_tab[j]];
      copy_row(prev_byp_src[j], prev_ovf + (size_t)j * st.stride, rb, lig);
      if (lig == 0) out_b += rb;
    }
  for (int i = group; i < n_ins; i += n_groups) {
    const int u = ins_idx[i];
    const TableMeta &m = tm[ins_tab[i]];
    const int slot = loc_u[u];
    const int32_t old = old_tag[u];
    const uint32_t rb = m.row_bytes;
    char *line = m.lines + (size_t)(slot - m.slot_base) * rb;
    const bool late = ins_late[i] != 0;
    const char *src = st.in + (size_t)i * st.stride;
    bool from_host = false;
    if (late) {
      const int j = find_key(prev_byp_key, n_prev, ins_key[i]);
      from_host = j < 0;
      src = j >= 0 ? prev_ovf + (size_t)j * st.stride : ins_src[i];
    }
    char *park = st.out + (size_t)i * st.stride;
    for (uint32_t c = lig * 16; c < rb; c += kMoveLanes * 16) {
      const uint4 fresh = *(const uint4 *)(src + c);
      if (old >= 0) *(uint4 *)(park + c) = *(const uint4 *)(line + c);
      *(uint4 *)(line + c) = fresh;
    }
    if (lig == 0) {
      if (old >= 0) {
        st.wb_dst[i] = m.host_w + (size_t)old * rb;
        st.wb_rb[i] = rb;
      } else {
        st.wb_dst[i] = nullptr;
      }
      if (from_host) in_b += rb;
    }
  }
  for (int j = group; j < n_byp; j += n_groups) {  // late bypassed rows
    if (byp_late[j] == 0) continue;
    const uint32_t rb = rb_of_table[byp_tab[j]];
    const int pj = find_key(prev_byp_key, n_prev, byp_key[j]);
    copy_row(ovf + (size_t)j * st.stride, pj >= 0 ? prev_ovf + (size_t)pj * st.stride : byp_src[j], rb, lig);
    if (lig == 0 && pj < 0) in_b += rb;
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
    copy_row(byp_src[j], ovf + (size_t)j * st.stride, rb, lig);
    if (lig == 0) out_b += rb;
  }
  for (int d = 32; d >= 1; d >>= 1) out_b += __shfl_xor(out_b, d);
  if ((threadIdx.x & 63) == 0 && out_b) atomicAdd(bytes_d2h, out_b);
}

hipError_t launch_ovf_writeback(const BatchBuf &b, const Staging &st, const uint32_t *rb_of_table, u64 *bytes_d2h,
                                hipStream_t s) {
  if (b.n == 0) return hipSuccess;
  hipLaunchKernelGGL(ovf_writeback_kernel, dim3(kLinkBlocks), dim3(256), 0, s, st, b.cnt, b.byp_src, b.byp_tab, b.ovf,
                     rb_of_table, bytes_d2h);
  return hipGetLastError();
}

hipError_t launch_commit(const TableMeta *tm, const BatchBuf &b, const BatchBuf *prev, bool wb_prev, const Staging &st,
                         const uint32_t *rb_of_table, u64 *bytes_h2d, u64 *bytes_d2h, hipStream_t s) {
  hipLaunchKernelGGL(commit_kernel, dim3(1024), dim3(256), 0, s, tm, st, b.cnt, b.ins_idx, b.ins_tab, b.ins_key,
                     b.ins_src, b.ins_late, b.loc_u, b.old_tag, b.byp_src, b.byp_tab, b.byp_key, b.byp_late, b.ovf,
                     prev ? prev->cnt : nullptr, prev ? prev->byp_key : nullptr, prev ? prev->byp_src : nullptr,
                     prev ? prev->byp_tab : nullptr, prev ? prev->ovf : nullptr, (prev && wb_prev) ? 1 : 0, rb_of_table,
                     bytes_h2d, bytes_d2h);
  return hipGetLastError();
}

// flush: every valid line goes to the backing tier (the accumulators are copied by the host code)
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
    copy_row(m.host_w + (size_t)row * m.row_bytes, m.lines + (size_t)(slot - m.slot_base) * m.row_bytes, m.row_bytes, lig);
    if (lig == 0) out_b += m.row_bytes;
  }
  for (int d = 32; d >= 1; d >>= 1) out_b += __shfl_xor(out_b, d);
  if ((threadIdx.x & 63) == 0 && out_b) atomicAdd(bytes_d2h, out_b);
}

hipError_t launch_flush(const TableMeta *tm, const Geometry &g, const int32_t *tags, u64 *bytes_d2h, hipStream_t s) {
  if (g.total_slots == 0) return hipSuccess;
  hipLaunchKernelGGL(flush_kernel, dim3(1024), dim3(256), 0, s, tm, g.T, g.total_slots, tags, bytes_d2h);
  return hipGetLastError();
}

}  // namespace tbe
