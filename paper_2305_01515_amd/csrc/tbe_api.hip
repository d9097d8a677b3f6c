// C ABI of libtbe: handle life cycle, the three-stream batch pipeline (compute, prefetch,
// host link), observation calls.
// Declarations and the contract of every call are in include/tbe.h.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <deque>
#include <mutex>
#include <vector>

#include "../../include/tbe.h"
#include "tbe_internal.h"

using namespace tbe;

// Scratch memory of tbe_backward_update_static: the partial sums of the backward's longest rows, for callers
// that must not allocate.  One copy per GPU, at an address of its own, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels are given the address it returns.
constexpr size_t kStaticScratchBytes = (size_t)TBE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_create_error;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on every GPU the library has been used on

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
hipError_t static_scratch_of_current_device(void **out, int *device) {
  *out = nullptr;
  hipError_t e = hipGetDevice(device);
  if (e != hipSuccess) return e;
  if (*device < 0 || *device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[*device]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[*device] = p;
  }
  *out = g_scratch_ptr[*device];
  return hipSuccess;
}

struct DevAlloc {  // everything hipMalloc'ed, freed together
  std::vector<void *> ptrs;
  template <class P>
  hipError_t get(P **p, size_t bytes) {
    void *v = nullptr;
    hipError_t e = hipMalloc(&v, bytes ? bytes : 16);
    if (e == hipSuccess) ptrs.push_back(v);
    *p = (P *)v;
    return e;
  }
  void release() {
    for (void *p : ptrs) (void)hipFree(p);
    ptrs.clear();
  }
};

}  // namespace

// Batch buffers rotate over three: the buffer of batch k is still read after k has trained
// (its bypass list by the commit of batch k+1) while batch k+2 is already being prefetched.
// A pipeline D batches deep (tbe_set_prefetch_depth) rotates over 2 D + 1: the overflow copies of batch k are
// read before the forward of every batch up to k + D, and batch k + 2 D + 1 may be prefetched once batch k + D
// has trained.
constexpr int kBatchBufs = 3;

struct tbe_ctx {
  Geometry g{};
  std::vector<TableMeta> tm;  // host copy
  TableMeta *d_tm = nullptr;
  ClassInfo ci{};
  DevAlloc mem;
  int32_t *tags = nullptr, *ts = nullptr, *freq = nullptr;
  int policy = TBE_POLICY_LRU;
  int pooling = TBE_POOL_SUM;
  DeferredInit di;              // deferred initialisation on read (off unless enabled)
  Throttle throttle;            // emulated slower backing tier (off unless tbe_set_backing_throttle was called)
  uint32_t *init_bits = nullptr;
  size_t huge_slots = 0;        // (huge row, bag range) pairs a batch can have
  Level2 l2;                    // second-level cache (off unless tbe_enable_second_level was called)
  char *lines2 = nullptr;       // its lines: one pinned host allocation
  unsigned long long *d_l2tot = nullptr;  // running totals of the four second-level counters
  float *d_state = nullptr;   // row-wise Adagrad accumulators of all rows of all tables
  float *d_slot_m = nullptr;  // ... and of the rows in the cache lines, by slot
  float *partials = nullptr;  // segment sums of the backward's longest rows
  float *static_partials = nullptr;  // the same in the library's static scratch array on this handle's GPU
  int device = -1;                   // GPU the handle was created on
  char *lines = nullptr;
  BatchBuf buf[kMaxBatchBufs]{};
  int nbuf = kBatchBufs;        // batch buffers in use
  int deep = 0;                 // 0: the one-deep pipeline; D >= 2: batches are fetched into the cache up to D ahead
  hipEvent_t ev_home[kMaxBatchBufs] = {};   // deep pipeline: the write-back of the buffer's bypassed rows
  bool home_pending[kMaxBatchBufs] = {};    // ... has been enqueued and the rows' marks are still in the map
  bool home_recorded[kMaxBatchBufs] = {};
  SortScratch ss{};
  Staging st{};
  uint32_t *d_rb = nullptr;  // row bytes of every table
  int prev_buf = -1;         // buffer of the batch prefetched before the current one
  BatchCounters *d_total = nullptr;       // running totals of the per-batch counters
  unsigned long long *d_bytes = nullptr;  // [0] backing->cache, [1] cache->backing
  hipStream_t cs = nullptr, as = nullptr;  // compute / prefetch streams (caller's)
  hipStream_t ls = nullptr;                // host-link stream: transfer and commit (own, unless cs == as)
  bool own_ls = false;

  hipEvent_t ev_fwd = nullptr;  // the last forward launched
  bool fwd_recorded = false;
  int last_trained = -1;        // buffer of the batch whose backward was launched last
  hipEvent_t ev_inputs = nullptr, ev_ready[kMaxBatchBufs] = {}, ev_trained[kMaxBatchBufs] = {}, ev_probed[kMaxBatchBufs] = {};
  int64_t flush_state_bytes = 0;
  bool inputs_ready = false;  // caller guarantees index / offset buffers are complete when tbe_prefetch is called
  int32_t max_batch = 0;
  int64_t max_lookups = 0;
  int32_t k = 0;
  // pipeline: buffers prefetched and waiting for forward (oldest first), the buffer that
  // was forwarded and waits for its update, and a buffer whose copies wait for that update
  int pend[kMaxBatchBufs] = {-1, -1};
  // batches accepted by tbe_prefetch further ahead than the pipeline runs: their work is issued, in order, as
  // soon as the batch before has been forwarded
  struct Queued { const int64_t *d_indices, *d_offsets; int32_t batch; int64_t n; };
  std::deque<Queued> queued;
  int depth = 1;                // batches tbe_prefetch accepts ahead of training (those beyond the next one are queued)
  int n_pend = 0;
  int current = -1;
  int deferred = -1;
  int last_buf = -1;
  int64_t total_lookups = 0;
  int sticky = 0;
  std::string err;
  // optional stage timing: (start, stop) event pairs per stage, in call order
  int profiling = 0;  // 0 off, 1 every bracket, 2 the whole-stage brackets only
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof[TBE_NUM_STAGES];
};

namespace {

int fail(tbe_ctx *h, int code, const std::string &msg) {
  if (h) h->err = msg; else g_create_error = msg;
  return code;
}

int hipfail(tbe_ctx *h, hipError_t e, const char *what) {
  (void)hipGetLastError();  // HIP keeps the error until it is read: the next launch check must not report it again
  return fail(h, e == hipErrorOutOfMemory ? TBE_ENOMEM : TBE_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define HIP_TRY(h, call)                                  \
  do {                                                    \
    hipError_t e__ = (call);                              \
    if (e__ != hipSuccess) return hipfail(h, e__, #call); \
  } while (0)

constexpr size_t kMaxProfiledCalls = 16384;

// Brackets the launches of one stage with timing events on the stream they go to.
struct StageTimer {
  tbe_ctx *h;
  hipStream_t s;
  hipEvent_t stop = nullptr;
  StageTimer(tbe_ctx *h_, int stage, hipStream_t s_) : h(h_), s(s_) {
    const bool inner = stage == TBE_STAGE_BACKWARD_HEAVY || stage == TBE_STAGE_BACKWARD_COMBINE ||
                       stage == TBE_STAGE_BACKWARD_SINGLE || stage == TBE_STAGE_BACKWARD_SHORT;
    if (!h->profiling || (inner && h->profiling == 2) || h->prof[stage].size() >= kMaxProfiledCalls) return;
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { if (a) (void)hipEventDestroy(a); return; }
    (void)hipEventRecord(a, s);
    h->prof[stage].emplace_back(a, b);
    stop = b;
  }
  ~StageTimer() { if (stop) (void)hipEventRecord(stop, s); }
};

void drop_profile(tbe_ctx *h) {
  for (auto &v : h->prof) {
    for (auto &p : v) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
    v.clear();
  }
}

int next_pow2(int v) { int p = 1; while (p < v) p <<= 1; return p; }

__global__ void stream_pin_kernel() {}

// Running totals of a batch's counters: tot (hits, evictions, lookups that hit), t64 ([0] distinct
// rows, [1] inserts, [2] bypasses) and, with a second level, l2 (its four counters).
// Also completes the batch's own counters: evictions and lookups that hit from the per-wavefront sums of the
// status pass (tens of thousands of them at the benchmark's batch: a single wavefront took 27 us to add them up),
// hits as what is left of the distinct rows.  One workgroup of kTotalsThreads.
constexpr int kTotalsThreads = 256;
__global__ __launch_bounds__(kTotalsThreads) void add_totals_kernel(BatchCounters *c, BatchCounters *tot,
                                                                    unsigned long long *t64, unsigned long long *l2,
                                                                    const unsigned long long *tally, int tally_waves) {
  if (c->err != 0) return;
  __shared__ unsigned long long s_e[kTotalsThreads / 64], s_l[kTotalsThreads / 64];
  unsigned long long e = 0, l = 0;
  for (int w = threadIdx.x; w < tally_waves; w += kTotalsThreads) { e += tally[2 * w]; l += tally[2 * w + 1]; }
  for (int d = 32; d >= 1; d >>= 1) { e += __shfl_xor(e, d); l += __shfl_xor(l, d); }
  if ((threadIdx.x & 63) == 0) { s_e[threadIdx.x >> 6] = e; s_l[threadIdx.x >> 6] = l; }
  __syncthreads();
  if (threadIdx.x != 0) return;
  e = l = 0;
  for (int w = 0; w < kTotalsThreads / 64; w++) { e += s_e[w]; l += s_l[w]; }
  c->hits = (unsigned long long)(c->n_uniq - c->n_ins - c->n_byp);
  c->evictions = e;
  c->hit_lookups = l;
  tot->hits += c->hits;
  tot->evictions += c->evictions;
  tot->hit_lookups += c->hit_lookups;
  t64[0] += (unsigned long long)c->n_uniq;
  t64[1] += (unsigned long long)c->n_ins;
  t64[2] += (unsigned long long)c->n_byp;
  if (l2) {
    l2[0] += (unsigned long long)c->l2_hits;
    l2[1] += (unsigned long long)c->l2_demotions;
    l2[2] += (unsigned long long)c->l2_evictions;
    l2[3] += (unsigned long long)c->l2_bypasses;
  }
}

int alloc_batchbuf(tbe_ctx *h, BatchBuf &b, int64_t n) {
  const size_t N = (size_t)std::max<int64_t>(n, 1);
  HIP_TRY(h, h->mem.get(&b.loc, 4 * N));
  HIP_TRY(h, h->mem.get(&b.sorted_bag, 4 * N));
  HIP_TRY(h, h->mem.get(&b.bag_of_pos, 4 * N));
  HIP_TRY(h, h->mem.get(&b.inv_len, 4 * (size_t)h->g.T * (size_t)h->max_batch));
  HIP_TRY(h, h->mem.get(&b.uid_sorted, 4 * N));
  HIP_TRY(h, h->mem.get(&b.uniq_key, 4 * N));
  HIP_TRY(h, h->mem.get(&b.run_off, 4 * (N + 1)));
  HIP_TRY(h, h->mem.get(&b.uniq_sid, 4 * N));
  HIP_TRY(h, h->mem.get(&b.uniq_tab, 4 * N));
  HIP_TRY(h, h->mem.get(&b.loc_u, 4 * N));
  HIP_TRY(h, h->mem.get(&b.status, N));
  HIP_TRY(h, h->mem.get(&b.old_tag, 4 * N));
  HIP_TRY(h, h->mem.get(&b.touched, 8 * N));
  HIP_TRY(h, h->mem.get(&b.ins_idx, 4 * N));
  HIP_TRY(h, h->mem.get(&b.ins_tab, 4 * N));
  HIP_TRY(h, h->mem.get(&b.ins_slot, 4 * N));
  HIP_TRY(h, h->mem.get(&b.ins_old, 4 * N));
  HIP_TRY(h, h->mem.get(&b.ins_key, 4 * N));
  HIP_TRY(h, h->mem.get(&b.ins_src, 8 * N));
  HIP_TRY(h, h->mem.get(&b.ins_where, 4 * N));
  HIP_TRY(h, h->mem.get(&b.byp_idx, 4 * N));
  HIP_TRY(h, h->mem.get(&b.byp_tab, 4 * N));
  HIP_TRY(h, h->mem.get(&b.byp_key, 4 * N));
  HIP_TRY(h, h->mem.get(&b.byp_src, 8 * N));
  HIP_TRY(h, h->mem.get(&b.byp_where, 4 * N));
  HIP_TRY(h, h->mem.get(&b.ovf, N * (size_t)h->g.ovf_stride));
  HIP_TRY(h, h->mem.get(&b.mid_idx, 4 * (N / 2 + 1)));
  HIP_TRY(h, h->mem.get(&b.heavy, 4 * (N / 32 + 1)));  // rows: N / 65 at most; extra parts: N / kHeavySplit at most
  HIP_TRY(h, h->mem.get(&b.heavy_sub, 4 * (N / 32 + 1)));
  HIP_TRY(h, h->mem.get(&b.harrive, 4 * (N / 32 + 1)));
  HIP_TRY(h, hipMemset(b.harrive, 0, 4 * (N / 32 + 1)));
  HIP_TRY(h, h->mem.get(&b.hchunks, 16 * (N / 32 + (size_t)h->g.T + 1)));
  HIP_TRY(h, h->mem.get(&b.hg_count, 4 * 2 * ((size_t)h->g.T + 1)));
  HIP_TRY(h, hipMemset(b.hg_count, 0, 4 * 2 * ((size_t)h->g.T + 1)));
  HIP_TRY(h, h->mem.get(&b.hperm, 4 * (N / 32 + 1)));
  HIP_TRY(h, h->mem.get(&b.hstart, 4 * (h->huge_slots + 1)));
  HIP_TRY(h, h->mem.get(&b.cnt, sizeof(BatchCounters)));
  HIP_TRY(h, hipMemset(b.cnt, 0, sizeof(BatchCounters)));
  return TBE_OK;
}

int device_error_code(int e) { return e == 0 ? 0 : e == 1 ? TBE_EINVAL : TBE_ERANGE; }

// After a synchronisation: pick up errors the device recorded.
int collect_device_errors(tbe_ctx *h) {
  for (int i = 0; i < h->nbuf; i++) {
    BatchCounters c;
    HIP_TRY(h, hipMemcpy(&c, h->buf[i].cnt, sizeof(c), hipMemcpyDeviceToHost));
    if (c.err && !h->sticky) {
      h->sticky = device_error_code(c.err);
      h->err = c.err == 1 ? "offsets are not a non-decreasing partition of [0, num_lookups]"
                          : "an index is outside its table";
    }
  }
  return h->sticky;
}

int sync_all(tbe_ctx *h) {
  HIP_TRY(h, hipStreamSynchronize(h->as));
  HIP_TRY(h, hipStreamSynchronize(h->ls));
  HIP_TRY(h, hipStreamSynchronize(h->cs));
  return TBE_OK;
}

// Victims of batch `bi` to the staging area, its new rows into the cache lines; then the
// batch is ready for forward.  Must follow the update of the batch before it.
int enqueue_commit(tbe_ctx *h, int bi, bool wb_prev) {
  BatchBuf &b = h->buf[bi];
  {
    StageTimer tm_(h, TBE_STAGE_COMMIT, h->ls);
    const int prev_mode = !wb_prev ? kPrevKeep : b.parks_prev ? kPrevPark : kPrevWrite;
    HIP_TRY(h, launch_commit(h->d_tm, b, b.prev_bi >= 0 ? &h->buf[b.prev_bi] : nullptr, prev_mode, h->st, h->l2, h->d_rb,
                             h->d_bytes + 1, false, h->ls));
  }
  HIP_TRY(h, hipEventRecord(h->ev_ready[bi], h->ls));
  return TBE_OK;
}

// Pipeline several batches deep (Section 5.7): the batch is fetched into the cache as soon as it is decided on.
// The ways of the batches that may still wait for their training are locked (ts >= k - D), so its victims and
// the lines it fills are used by none of them and nothing waits for a backward -- except the rows whose current
// value is an overflow copy of such a batch: they are copied before this batch's forward (launch_fixup).
int do_prefetch_deep(tbe_ctx *h, const int64_t *d_indices, const int64_t *d_offsets, int32_t batch, int64_t n) {
  if (h->n_pend + (h->current >= 0 ? 1 : 0) > h->deep)
    return fail(h, TBE_EORDER, "prefetch: more batches would be ahead of training than the prefetch depth");
  const int bi = h->k % h->nbuf;
  BatchBuf &b = h->buf[bi];
  b.d_indices = d_indices; b.d_offsets = d_offsets; b.batch = batch; b.n = n; b.k = ++h->k;
  b.mean = h->pooling == TBE_POOL_MEAN;
  b.maxp = h->pooling == TBE_POOL_MAX;
  b.parks_prev = false;
  h->total_lookups += n;
  h->last_buf = bi;
  if (h->as != h->cs) {
    if (!h->inputs_ready) {
      HIP_TRY(h, hipEventRecord(h->ev_inputs, h->cs));
      HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_inputs, 0));
    } else {
      if (h->fwd_recorded) HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_fwd, 0));
    }
    // the buffer last served batch k - (2 D + 1): every batch that read its overflow copies (up to k - D - 1) has
    // trained, and its bypassed rows have been written back
    if (h->last_trained >= 0) HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_trained[h->last_trained], 0));
    if (h->home_recorded[bi]) HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_home[bi], 0));
  }
  {
    StageTimer tm_(h, TBE_STAGE_PREFETCH, h->as);
    // batches whose bypassed rows are on their way home in front of this batch's transfer: their marks go
    // (before this buffer's lists are overwritten, should it be one of them)
    for (int x = 0; x < h->nbuf; x++)
      if (h->home_pending[x]) {
        HIP_TRY(h, launch_unmark_bypassed(h->buf[x], x, h->st, h->as));
        h->home_pending[x] = false;
      }
    HIP_TRY(h, launch_keygen(h->d_tm, h->g, b, h->ss.keys[0], h->ss.vals[0], h->as));
    int res = 0;
    HIP_TRY(h, launch_sort(h->g, h->ss, n, &res, h->as));
    HIP_TRY(h, launch_dedup_probe(h->d_tm, h->g, b, h->ss, h->ss.keys[res], h->ss.vals[res], h->tags, h->ts, h->freq,
                                  h->policy == TBE_POLICY_LFU, h->l2, h->deep, h->as));
    const BatchBuf *prev = h->prev_buf >= 0 ? &h->buf[h->prev_buf] : nullptr;
    HIP_TRY(h, launch_classify_mark_deep(h->d_tm, prev, b, bi, h->st, h->d_bytes + 5, h->as));
    hipLaunchKernelGGL(add_totals_kernel, dim3(1), dim3(kTotalsThreads), 0, h->as, b.cnt, h->d_total, h->d_bytes + 2,
                       (unsigned long long *)nullptr, h->ss.tally, n > 0 ? h->ss.tally_waves : 0);
    HIP_TRY(h, hipGetLastError());
  }
  if (h->ls != h->as) {
    HIP_TRY(h, hipEventRecord(h->ev_probed[bi], h->as));
    HIP_TRY(h, hipStreamWaitEvent(h->ls, h->ev_probed[bi], 0));
  }
  {
    StageTimer tm_(h, TBE_STAGE_FILL, h->ls);
    HIP_TRY(h, launch_transfer(&b, h->st, h->l2, h->di, h->throttle, b.k, h->d_rb, h->d_bytes, h->d_bytes + 1, h->ls));
  }
  b.prev_bi = h->prev_buf;
  h->prev_buf = bi;
  h->pend[h->n_pend++] = bi;
  {
    // the link stream waits for every backward launched so far (tbe_backward_update sees to that), which covers the
    // batches whose lines this commit may overwrite: they were stamped before k - D
    StageTimer tm_(h, TBE_STAGE_COMMIT, h->ls);
    HIP_TRY(h, launch_commit(h->d_tm, b, nullptr, kPrevKeep, h->st, h->l2, h->d_rb, h->d_bytes + 1, true, h->ls));
  }
  HIP_TRY(h, hipEventRecord(h->ev_ready[bi], h->ls));
  return TBE_OK;
}

int do_prefetch(tbe_ctx *h, const int64_t *d_indices, const int64_t *d_offsets, int32_t batch, int64_t n) {
  if (!d_offsets || batch < 0 || n < 0 || (n > 0 && !d_indices)) return fail(h, TBE_EINVAL, "prefetch: bad argument");
  if (batch > h->max_batch || n > h->max_lookups) return fail(h, TBE_ELIMIT, "prefetch: batch or lookups above the sizes given to tbe_create");
  if (h->deep) return do_prefetch_deep(h, d_indices, d_offsets, batch, n);
  if (h->n_pend + (h->current >= 0 ? 1 : 0) > 1) return fail(h, TBE_EORDER, "prefetch: more than one batch would be ahead of training");
  const int bi = h->k % kBatchBufs;  // free: at most the batch before this one is still in use
  BatchBuf &b = h->buf[bi];
  const bool in_flight = h->n_pend > 0 || h->current >= 0;
  b.d_indices = d_indices; b.d_offsets = d_offsets; b.batch = batch; b.n = n; b.k = ++h->k;
  b.mean = h->pooling == TBE_POOL_MEAN;
  b.maxp = h->pooling == TBE_POOL_MAX;
  // A batch prefetched while its predecessor is still in flight is committed right after that one's
  // update, and its commit then parks the predecessor's overflow copies for the next transfer.
  b.parks_prev = in_flight && h->prev_buf >= 0 && h->st.max_parked > 0 && !h->l2.on;
  h->total_lookups += n;
  h->last_buf = bi;
  if (h->as != h->cs) {
    if (!h->inputs_ready) {  // inputs produced on the compute stream so far come first
      HIP_TRY(h, hipEventRecord(h->ev_inputs, h->cs));
      HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_inputs, 0));
    } else {
      // Training launched so far goes first: its kernels and this stage are all bound by HBM and slow each
      // other down when they overlap, the model waits for training, and this stage has the whole transfer of
      // the batch before it to finish in.  (Benchmark workload, this stage behind the last forward only, i.e.
      // beside the backward: forward 0.27 ms, backward 0.78 ms, this stage 1.5 ms per step; behind both: see
      // the design notes.  The step is bound by the host link either way.)
      if (h->fwd_recorded) HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_fwd, 0));
      if (h->last_trained >= 0) HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_trained[h->last_trained], 0));
    }
    // this buffer last served the batch three before: its backward read the buffer's arrays,
    // and the commit of the batch after it read its bypass list and overflow copies
    HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_trained[bi], 0));
    HIP_TRY(h, hipStreamWaitEvent(h->as, h->ev_ready[(bi + 1) % kBatchBufs], 0));
  }
  {
    StageTimer tm_(h, TBE_STAGE_PREFETCH, h->as);
    HIP_TRY(h, launch_keygen(h->d_tm, h->g, b, h->ss.keys[0], h->ss.vals[0], h->as));
    int res = 0;
    HIP_TRY(h, launch_sort(h->g, h->ss, n, &res, h->as));
    HIP_TRY(h, launch_dedup_probe(h->d_tm, h->g, b, h->ss, h->ss.keys[res], h->ss.vals[res], h->tags, h->ts, h->freq,
                                  h->policy == TBE_POLICY_LFU, h->l2, 0, h->as));
    // which of the rows to insert have a backing-tier copy that is still being written
    // (by the write-back of the previous batch's victims or by its backward), then move
    // the marks on from the previous batch to this one
    const BatchBuf *prev = h->prev_buf >= 0 ? &h->buf[h->prev_buf] : nullptr;
    const BatchBuf *pp = (prev && prev->parks_prev && prev->prev_bi >= 0) ? &h->buf[prev->prev_bi] : nullptr;
    HIP_TRY(h, launch_classify_mark(h->d_tm, pp, prev, b, h->st, h->l2, h->d_bytes + 5, h->as));
    hipLaunchKernelGGL(add_totals_kernel, dim3(1), dim3(kTotalsThreads), 0, h->as, b.cnt, h->d_total, h->d_bytes + 2,
                       h->l2.on ? h->d_l2tot : nullptr, h->ss.tally, n > 0 ? h->ss.tally_waves : 0);
    HIP_TRY(h, hipGetLastError());
  }
  if (h->ls != h->as) {
    HIP_TRY(h, hipEventRecord(h->ev_probed[bi], h->as));
    HIP_TRY(h, hipStreamWaitEvent(h->ls, h->ev_probed[bi], 0));
  }
  {
    // write-back of the previous batch's victims and fetch-ahead of this batch's rows share
    // the host link; neither touches a cache line, so a batch in flight is not disturbed,
    // and the link stream lets the next batch's sort and probe run meanwhile
    StageTimer tm_(h, TBE_STAGE_FILL, h->ls);
    HIP_TRY(h, launch_transfer(&b, h->st, h->l2, h->di, h->throttle, b.k, h->d_rb, h->d_bytes, h->d_bytes + 1, h->ls));
  }
  b.prev_bi = h->prev_buf;
  h->prev_buf = bi;
  h->pend[h->n_pend++] = bi;
  if (in_flight) {
    h->deferred = bi;  // its cache lines may still be in use: commit after that batch's update
    return TBE_OK;
  }
  return enqueue_commit(h, bi, false);
}

}  // namespace

extern "C" {

const char *tbe_last_error(tbe_handle h) { return h ? h->err.c_str() : g_create_error.c_str(); }

int tbe_host_alloc(void **h_ptr, size_t bytes) {
  if (!h_ptr) return TBE_EINVAL;
  hipError_t e = hipHostMalloc(h_ptr, bytes ? bytes : 16, hipHostMallocDefault);
  if (e != hipSuccess) { *h_ptr = nullptr; (void)hipGetLastError(); return TBE_ENOMEM; }
  return TBE_OK;
}

int tbe_host_free(void *h_ptr) { return hipHostFree(h_ptr) == hipSuccess ? TBE_OK : TBE_EHIP; }

int tbe_destroy(tbe_handle h) {
  if (!h) return TBE_EINVAL;
  (void)hipStreamSynchronize(h->as);
  (void)hipStreamSynchronize(h->ls);
  (void)hipStreamSynchronize(h->cs);
  if (h->own_ls) (void)hipStreamDestroy(h->ls);
  h->mem.release();
  if (h->lines2) (void)hipHostFree(h->lines2);
  drop_profile(h);
  if (h->ev_inputs) (void)hipEventDestroy(h->ev_inputs);
  if (h->ev_fwd) (void)hipEventDestroy(h->ev_fwd);
  for (int i = 0; i < kMaxBatchBufs; i++) {
    if (h->ev_ready[i]) (void)hipEventDestroy(h->ev_ready[i]);
    if (h->ev_trained[i]) (void)hipEventDestroy(h->ev_trained[i]);
    if (h->ev_probed[i]) (void)hipEventDestroy(h->ev_probed[i]);
    if (h->ev_home[i]) (void)hipEventDestroy(h->ev_home[i]);
  }
  delete h;
  return TBE_OK;
}

int tbe_create(tbe_handle *out, const tbe_table_spec *specs, int32_t num_tables, int32_t ways, int32_t max_batch,
               int64_t max_lookups, void *compute_stream, void *aux_stream) {
  if (!out) return fail(nullptr, TBE_EINVAL, "create: null output handle");
  *out = nullptr;
  if (!specs || num_tables <= 0) return fail(nullptr, TBE_EINVAL, "create: no tables");
  if (ways < 1 || ways > kWave) return fail(nullptr, TBE_EINVAL, "create: ways must be 1..64");
  if (max_batch < 1 || max_lookups < 1 || max_lookups > (1ll << 30))
    return fail(nullptr, TBE_EINVAL, "create: max_batch >= 1 and 1 <= max_lookups <= 2^30 required");
  if ((int64_t)num_tables * max_batch >= (1ll << 31)) return fail(nullptr, TBE_ELIMIT, "create: tables x batch too large");
  tbe_ctx *h = new (std::nothrow) tbe_ctx();
  if (!h) return fail(nullptr, TBE_ENOMEM, "create: host allocation failed");
  h->cs = (hipStream_t)compute_stream;
  h->as = (hipStream_t)aux_stream;
  h->ls = h->cs;
  h->max_batch = max_batch;
  h->max_lookups = max_lookups;
  h->g.T = num_tables;
  h->g.ways = ways;
  h->tm.resize(num_tables);
  uint64_t key = 0, sets = 0;
  int64_t col = 0;
  size_t line_bytes = 0;
  std::vector<size_t> line_off(num_tables);
  std::vector<int> tclass(num_tables);
  for (int t = 0; t < num_tables; t++) {
    const tbe_table_spec &s = specs[t];
    TableMeta &m = h->tm[t];
    const int epl = s.dtype == TBE_FP32 ? 4 : 8;
    if ((s.dtype != TBE_FP32 && s.dtype != TBE_FP16) || s.rows < 1 || s.rows >= (1ll << 31) || s.dim < epl ||
        s.dim % epl || s.dim > 64 * epl || !s.host_weights || !s.host_state || s.cache_slots < 0) {
      delete h;
      return fail(nullptr, TBE_EINVAL, "create: bad table spec " + std::to_string(t));
    }
    m.rows = s.rows;
    m.dim = s.dim;
    m.dtype = s.dtype;
    m.row_bytes = (uint32_t)(s.dim * (s.dtype == TBE_FP32 ? 4 : 2));
    m.lanes = next_pow2(s.dim / epl);
    m.col = (int32_t)col;
    m.sets = (uint32_t)std::min<int64_t>(s.cache_slots / ways, (1ll << 31) / ways);
    m.rows_per_set = m.sets ? (uint32_t)((s.rows + m.sets - 1) / m.sets) : 0;
    m.key_base = (uint32_t)key;
    m.set_base = (uint32_t)sets;
    m.slot_base = (int32_t)(sets * ways);
    m.host_w = (char *)s.host_weights;
    m.host_m = s.host_state;
    key += m.sets ? (uint64_t)m.sets * m.rows_per_set : (uint64_t)s.rows;
    sets += m.sets;
    col += s.dim;
    line_off[t] = line_bytes;
    line_bytes += ((size_t)m.sets * ways * m.row_bytes + 255) & ~(size_t)255;
    if (key > (1ull << 32) || sets * ways >= (1ull << 30) || col >= (1ll << 30)) {
      delete h;
      return fail(nullptr, TBE_ELIMIT, "create: key space, slot count or output width too large");
    }
    // class of the table
    int c = 0;
    for (; c < h->ci.n_classes; c++)
      if (h->ci.cls_dtype[c] == m.dtype && h->ci.cls_lanes[c] == m.lanes) break;
    if (c == h->ci.n_classes) {
      h->ci.cls_dtype[c] = m.dtype;
      h->ci.cls_lanes[c] = m.lanes;
      h->ci.cls_count[c] = 0;
      h->ci.n_classes++;
    }
    h->ci.cls_count[c]++;
    tclass[t] = c;
  }
  h->g.sum_dim = (int32_t)col;
  h->g.total_sets = (uint32_t)sets;
  h->g.total_slots = (int64_t)sets * ways;
  h->g.ovf_stride = 16;
  for (const TableMeta &m : h->tm) h->g.ovf_stride = std::max(h->g.ovf_stride, m.row_bytes);
  h->g.key_bits = 1;
  while (h->g.key_bits < 32 && (1ull << h->g.key_bits) < key) h->g.key_bits++;
  {  // sort payload (bag, position inside the bag) when both fit 32 bits
    int bag_bits = 0;
    while ((1ll << bag_bits) < (int64_t)num_tables * max_batch) bag_bits++;
    h->g.within_bits = std::min(24, 32 - bag_bits);
    if (h->g.within_bits < 1) h->g.within_bits = 0;
  }

  auto bail = [&](int code) { tbe_destroy(h); return code; };
  auto hipbail = [&](hipError_t e, const char *what) {
    int code = hipfail(nullptr, e, what);
    tbe_destroy(h);
    return code;
  };
#define CREATE_TRY(call)                                  \
  do {                                                    \
    hipError_t e__ = (call);                              \
    if (e__ != hipSuccess) return hipbail(e__, #call);    \
  } while (0)

  const size_t slots = (size_t)h->g.total_slots;
  CREATE_TRY(h->mem.get(&h->lines, line_bytes));
  CREATE_TRY(h->mem.get(&h->tags, 4 * slots));
  CREATE_TRY(h->mem.get(&h->ts, 4 * slots));
  CREATE_TRY(h->mem.get(&h->freq, 4 * slots));
  if (slots) {
    CREATE_TRY(hipMemset(h->tags, 0xFF, 4 * slots));  // -1 = free
    CREATE_TRY(hipMemset(h->ts, 0xFF, 4 * slots));
    CREATE_TRY(hipMemset(h->freq, 0, 4 * slots));
  }
  {  // accumulators of all rows live in HBM; the host arrays give their initial values
    size_t total_rows = 0;
    for (int t = 0; t < num_tables; t++) total_rows += (size_t)h->tm[t].rows;
    CREATE_TRY(h->mem.get(&h->d_state, 4 * total_rows));
    size_t off = 0;
    for (int t = 0; t < num_tables; t++) {
      h->tm[t].dev_m = h->d_state + off;
      CREATE_TRY(hipMemcpy(h->tm[t].dev_m, h->tm[t].host_m, 4 * (size_t)h->tm[t].rows, hipMemcpyHostToDevice));
      off += (size_t)h->tm[t].rows;
    }
  }
  if (h->as != h->cs) {
    CREATE_TRY(hipStreamCreateWithFlags(&h->ls, hipStreamNonBlocking));
    h->own_ls = true;
  }
  CREATE_TRY(h->mem.get(&h->d_slot_m, 4 * slots));
  if (slots) CREATE_TRY(hipMemset(h->d_slot_m, 0, 4 * slots));
  for (int t = 0; t < num_tables; t++) {
    h->tm[t].lines = h->lines + line_off[t];
    h->tm[t].slot_m = h->d_slot_m + h->tm[t].slot_base;
  }
  CREATE_TRY(h->mem.get(&h->d_tm, sizeof(TableMeta) * num_tables));
  CREATE_TRY(hipMemcpy(h->d_tm, h->tm.data(), sizeof(TableMeta) * num_tables, hipMemcpyHostToDevice));
  {  // class tables
    int32_t *d_tc = nullptr;
    CREATE_TRY(h->mem.get(&d_tc, 4 * (size_t)num_tables));
    CREATE_TRY(hipMemcpy(d_tc, tclass.data(), 4 * (size_t)num_tables, hipMemcpyHostToDevice));
    h->ci.table_class = d_tc;
    for (int c = 0; c < h->ci.n_classes; c++) {
      std::vector<int32_t> ids;
      for (int t = 0; t < num_tables; t++)
        if (tclass[t] == c) ids.push_back(t);
      int32_t *d_ids = nullptr;
      CREATE_TRY(h->mem.get(&d_ids, 4 * ids.size()));
      CREATE_TRY(hipMemcpy(d_ids, ids.data(), 4 * ids.size(), hipMemcpyHostToDevice));
      h->ci.cls_tables[c] = d_ids;
    }
  }
  // (heavy-list entry, bag range) pairs of a batch, one partial sum each: a batch has at most N / 32 entries
  // (N / 65 heavy rows, N / kHeavySplit more for the parts of the hot ones); the number of ranges is chosen
  // per batch so that the pairs fit (heavy_ranges)
  h->huge_slots = std::max<size_t>(4 * ((size_t)max_lookups / (kLongRun + 1) + 1), 32768);
  h->g.partial_slots = (int64_t)h->huge_slots;
  {
    int dev = 0, cus = 256;
    (void)hipGetDevice(&dev);
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    (void)hipGetLastError();
    // the transfer kernel keeps kLinkCus CUs to itself while it runs, which is most of the time when the link has
    // a stream of its own and rows miss (the same figure without such a stream: the split of the sums, and with
    // it their rounding, must not depend on how the streams are arranged)
    h->g.heavy_target = std::max(8, cus - kLinkCus);
  }
  for (int i = 0; i < kBatchBufs; i++) {
    int rc = alloc_batchbuf(h, h->buf[i], max_lookups);
    if (rc) { g_create_error = h->err; return bail(rc); }
    CREATE_TRY(hipEventCreateWithFlags(&h->ev_ready[i], hipEventDisableTiming));
    CREATE_TRY(hipEventCreateWithFlags(&h->ev_trained[i], hipEventDisableTiming));
    CREATE_TRY(hipEventCreateWithFlags(&h->ev_probed[i], hipEventDisableTiming));
  }
  CREATE_TRY(hipEventCreateWithFlags(&h->ev_inputs, hipEventDisableTiming));
  CREATE_TRY(hipEventCreateWithFlags(&h->ev_fwd, hipEventDisableTiming));
  const size_t N = (size_t)max_lookups;
  for (int i = 0; i < 2; i++) {
    CREATE_TRY(h->mem.get(&h->ss.keys[i], 4 * N));
    CREATE_TRY(h->mem.get(&h->ss.vals[i], 4 * N));
  }
  {
    int widest = 0;
    for (const TableMeta &m : h->tm) widest = std::max(widest, m.lanes * (m.dtype == TBE_FP32 ? 4 : 8));
    h->g.partial_stride = widest;
    CREATE_TRY(h->mem.get(&h->partials, 4 * (size_t)widest * h->huge_slots));
  }
  {
    Staging &st = h->st;
    st.max_inserts = std::min<int64_t>(max_lookups, h->g.total_slots);
    st.stride = h->g.ovf_stride;
    std::vector<uint32_t> rb(num_tables);
    for (int t = 0; t < num_tables; t++) { rb[t] = h->tm[t].row_bytes; st.stride = std::max(st.stride, rb[t]); }
    const size_t M = (size_t)st.max_inserts;
    // room behind the victims for the overflow copies a commit parks with them (a batch bypasses at
    // most as many rows as it has lookups); none when the indices would not fit the map's codes
    st.max_parked = (M + (size_t)max_lookups <= (size_t)kWhereIndex) ? max_lookups : 0;
    const size_t P = M + (size_t)st.max_parked;
    CREATE_TRY(h->mem.get(&st.in, M * st.stride));
    for (int p2 = 0; p2 < 2; p2++) {
      CREATE_TRY(h->mem.get(&st.out[p2], P * st.stride));
      CREATE_TRY(h->mem.get(&st.wb_skip[p2], P));
      CREATE_TRY(hipMemset(st.wb_skip[p2], 0, P ? P : 1));
    }
    CREATE_TRY(h->mem.get(&st.wb_dst, 8 * P));
    CREATE_TRY(h->mem.get(&st.wb_rb, 4 * P));
    CREATE_TRY(h->mem.get(&st.wb_n, 16));
    CREATE_TRY(hipMemset(st.wb_n, 0, 16));
    CREATE_TRY(h->mem.get(&st.where, 4 * (size_t)key));
    CREATE_TRY(hipMemset(st.where, 0, 4 * (size_t)key));
    CREATE_TRY(h->mem.get(&h->d_rb, 4 * (size_t)num_tables));
    CREATE_TRY(hipMemcpy(h->d_rb, rb.data(), 4 * (size_t)num_tables, hipMemcpyHostToDevice));
  }
  {
    void *p = nullptr;
    CREATE_TRY(static_scratch_of_current_device(&p, &h->device));
    h->static_partials = (float *)p;
  }
  CREATE_TRY(h->mem.get(&h->ss.hist, 4 * (512 * 1024 + 512)));  // sort: counts per digit value (<= 512) and block (<= 1024), digit totals
  CREATE_TRY(h->mem.get(&h->ss.blk, 8 * (8192 + 1)));
  CREATE_TRY(h->mem.get(&h->ss.tally, 8 * 2 * 8192));
  CREATE_TRY(h->mem.get(&h->ss.wl, 4 * 4 * (size_t)kWorklistBlocks));
  CREATE_TRY(h->mem.get(&h->d_total, sizeof(BatchCounters)));
  CREATE_TRY(hipMemset(h->d_total, 0, sizeof(BatchCounters)));
  CREATE_TRY(h->mem.get(&h->d_bytes, 8 * 8));
  CREATE_TRY(hipMemset(h->d_bytes, 0, 8 * 8));
  CREATE_TRY(hipDeviceSynchronize());
#undef CREATE_TRY
  *out = h;
  return TBE_OK;
}

// issue the work of queued batches as far as the pipeline takes them (one batch ahead of training)
static int pump_queue(tbe_ctx *h) {
  while (!h->queued.empty() && h->n_pend + (h->current >= 0 ? 1 : 0) <= 1) {
    const tbe_ctx::Queued q = h->queued.front();
    h->queued.pop_front();
    int rc = do_prefetch(h, q.d_indices, q.d_offsets, q.batch, q.n);
    if (rc) return rc;
  }
  return TBE_OK;
}

int tbe_prefetch(tbe_handle h, const int64_t *d_indices, const int64_t *d_offsets, int32_t batch, int64_t num_lookups) {
  if (!h) return TBE_EINVAL;
  if (h->sticky) return h->sticky;
  const int ahead = h->n_pend + (h->current >= 0 ? 1 : 0) + (int)h->queued.size();
  if (h->depth > 1 && (ahead > 1 || !h->queued.empty())) {  // beyond what runs now: keep it for later
    if (!d_offsets || batch < 0 || num_lookups < 0 || (num_lookups > 0 && !d_indices)) return fail(h, TBE_EINVAL, "prefetch: bad argument");
    if (batch > h->max_batch || num_lookups > h->max_lookups) return fail(h, TBE_ELIMIT, "prefetch: batch or lookups above the sizes given to tbe_create");
    if (ahead > h->depth) return fail(h, TBE_EORDER, "prefetch: more batches ahead of training than the queue takes");
    h->queued.push_back({d_indices, d_offsets, batch, num_lookups});
    return TBE_OK;
  }
  return do_prefetch(h, d_indices, d_offsets, batch, num_lookups);
}

int tbe_set_prefetch_depth(tbe_handle h, int32_t depth) {
  if (!h) return TBE_EINVAL;
  if (depth < 1 || 2 * depth + 1 > kMaxBatchBufs) return fail(h, TBE_EINVAL, "set_prefetch_depth: depth must be 1..7");
  if (h->k != 0) return fail(h, TBE_EORDER, "set_prefetch_depth: batches have been prefetched already");
  if (h->deep) return fail(h, TBE_EORDER, "set_prefetch_depth: already set");
  if (depth == 1) return TBE_OK;  // the pipeline as it is
  if (h->l2.on) return fail(h, TBE_EORDER, "set_prefetch_depth: not together with a second level");
  if (h->depth != 1) return fail(h, TBE_EORDER, "set_prefetch_depth: not together with a prefetch queue");
  if (h->max_lookups > (int64_t)kWhereBufIndex) return fail(h, TBE_ELIMIT, "set_prefetch_depth: max_lookups must be below 2^26");
  const int want = 2 * depth + 1;
  for (int i = h->nbuf; i < want; i++) {
    int rc = alloc_batchbuf(h, h->buf[i], h->max_lookups);
    if (rc) return rc;
    if (h->pooling == TBE_POOL_MAX) {
      HIP_TRY(h, h->mem.get(&h->buf[i].argpos, 4 * (size_t)h->max_batch * (size_t)h->g.sum_dim));
      HIP_TRY(h, h->mem.get(&h->buf[i].sorted_within, 4 * (size_t)std::max<int64_t>(h->max_lookups, 1)));
    }
    HIP_TRY(h, hipEventCreateWithFlags(&h->ev_ready[i], hipEventDisableTiming));
    HIP_TRY(h, hipEventCreateWithFlags(&h->ev_trained[i], hipEventDisableTiming));
    HIP_TRY(h, hipEventCreateWithFlags(&h->ev_probed[i], hipEventDisableTiming));
    h->nbuf = i + 1;
  }
  for (int i = 0; i < want; i++) HIP_TRY(h, hipEventCreateWithFlags(&h->ev_home[i], hipEventDisableTiming));
  HIP_TRY(h, hipDeviceSynchronize());
  h->deep = depth;
  return TBE_OK;
}

int tbe_get_prefetch_depth(tbe_handle h, int32_t *depth, int64_t *rows_from_copies) {
  if (!h || !depth || !rows_from_copies) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  unsigned long long n = 0;
  HIP_TRY(h, hipMemcpy(&n, h->d_bytes + 6, sizeof(n), hipMemcpyDeviceToHost));
  *depth = h->deep ? h->deep : 1;
  *rows_from_copies = (int64_t)n;
  return TBE_OK;
}

int tbe_set_prefetch_queue(tbe_handle h, int32_t depth) {
  if (!h) return TBE_EINVAL;
  if (h->deep) return fail(h, TBE_EORDER, "set_prefetch_queue: not together with a prefetch depth above one");
  if (depth < 1 || depth > 64) return fail(h, TBE_EINVAL, "set_prefetch_queue: length must be 1..64");
  if (!h->queued.empty()) return fail(h, TBE_EORDER, "set_prefetch_queue: batches are queued");
  h->depth = depth;
  return TBE_OK;
}

int tbe_forward(tbe_handle h, const int64_t *d_indices, const int64_t *d_offsets, int32_t batch, int64_t num_lookups,
                float *d_out) {
  if (!h) return TBE_EINVAL;
  if (h->sticky) return h->sticky;
  if (!d_out) return fail(h, TBE_EINVAL, "forward: null output");
  if (h->current >= 0) return fail(h, TBE_EORDER, "forward: the previous batch has not been updated");
  if (h->n_pend == 0 && !h->queued.empty()) {
    int rc = pump_queue(h);
    if (rc) return rc;
  }
  if (h->n_pend == 0) {
    int rc = do_prefetch(h, d_indices, d_offsets, batch, num_lookups);
    if (rc) return rc;
  }
  const int bi = h->pend[0];
  BatchBuf &b = h->buf[bi];
  if (b.d_indices != d_indices || b.d_offsets != d_offsets || b.batch != batch || b.n != num_lookups)
    return fail(h, TBE_EMISMATCH, "forward: buffers differ from the pending prefetch");
  if (h->deferred == bi) return fail(h, TBE_EORDER, "forward: the batch before this one has not been updated");
  for (int i = 1; i < h->n_pend; i++) h->pend[i - 1] = h->pend[i];
  h->n_pend--;
  if (h->as != h->cs) {
    HIP_TRY(h, hipStreamWaitEvent(h->cs, h->ev_ready[bi], 0));
    // A timing event recorded right after a wait for another stream is stamped before that wait is
    // over (measured: the forward's bracket began 0.15 ms before the commit it waits for had ended).
    // A kernel is held back by the wait, so an empty one in front of the bracket pins its beginning.
    if (h->profiling) hipLaunchKernelGGL(stream_pin_kernel, dim3(1), dim3(64), 0, h->cs);
  }
  if (h->deep) {  // rows whose value was an overflow copy of a batch that had not trained when this one was fetched
    OverflowCopies oc{};
    for (int x = 0; x < h->nbuf; x++) oc.of_buf[x] = h->buf[x].ovf;
    HIP_TRY(h, launch_fixup(h->d_tm, b, oc, h->st, h->d_rb, h->d_bytes + 6, h->cs));
  }
  {
    StageTimer tm_(h, TBE_STAGE_FORWARD, h->cs);
    HIP_TRY(h, launch_forward_classes(h->d_tm, h->ci, h->g, b, d_out, h->cs));
  }
  if (h->as != h->cs) {
    HIP_TRY(h, hipEventRecord(h->ev_fwd, h->cs));
    h->fwd_recorded = true;
  }
  h->current = bi;
  return pump_queue(h);  // the next queued batch is prefetched while this one trains
}

// The backward of the forwarded batch with the partial sums of its longest rows in `partials`.
static int backward_update_with(tbe_ctx *h, const float *d_grad_out, float lr, float eps, float *partials) {
  if (h->sticky) return h->sticky;
  if (!d_grad_out) return fail(h, TBE_EINVAL, "backward_update: null gradient");
  if (h->current < 0) return fail(h, TBE_EORDER, "backward_update: no forwarded batch");
  const int bi = h->current;
  // The four kernels touch disjoint rows and run one after the other.  (The heavy rows' tile kernel and its
  // combine on a stream of their own, beside the other two: the tile kernel's workgroups need a CU to
  // themselves each and waited for the others' waves to drain -- 0.28 ms instead of 0.12 alone, the whole
  // backward 0.51 ms instead of 0.48, and 0.72 instead of 0.65 ms beside the other streams' work.)
  {
    StageTimer all_(h, TBE_STAGE_BACKWARD, h->cs);
    auto heavy = [&]() -> int {
      {
        StageTimer tm_(h, TBE_STAGE_BACKWARD_HEAVY, h->cs);
        HIP_TRY(h, launch_backward_classes(kBwdHeavy, h->d_tm, h->ci, h->g, h->buf[bi], d_grad_out, partials, lr, eps, h->cs));
      }
      StageTimer tm_(h, TBE_STAGE_BACKWARD_COMBINE, h->cs);
      HIP_TRY(h, launch_backward_classes(kBwdCombine, h->d_tm, h->ci, h->g, h->buf[bi], d_grad_out, partials, lr, eps, h->cs));
      return TBE_OK;
    };
    auto single = [&]() -> int {
      StageTimer tm_(h, TBE_STAGE_BACKWARD_SINGLE, h->cs);
      HIP_TRY(h, launch_backward_single_classes(h->d_tm, h->ci, h->g, h->buf[bi], d_grad_out, lr, eps, h->cs));
      return TBE_OK;
    };
    auto shortk = [&]() -> int {
      StageTimer tm_(h, TBE_STAGE_BACKWARD_SHORT, h->cs);
      HIP_TRY(h, launch_backward_classes(kBwdShort, h->d_tm, h->ci, h->g, h->buf[bi], d_grad_out, partials, lr, eps, h->cs));
      return TBE_OK;
    };
    // single-lookup rows first, the heavy rows' tile kernel last: 0.471 ms alone against 0.479 with the tile kernel
    // first (it takes 0.124 instead of 0.134 ms when it does not follow the forward), 0.627 against 0.635 ms beside
    // the other streams; the other orders lie between
    int rc;
    if ((rc = single()) || (rc = shortk()) || (rc = heavy())) return rc;
  }
  h->current = -1;
  if (h->as != h->cs) {
    HIP_TRY(h, hipEventRecord(h->ev_trained[bi], h->cs));
    h->last_trained = bi;
    // later commits overwrite lines this batch used (the prefetch stream only decides on
    // tags and timestamps, which training never reads, so it does not wait here)
    HIP_TRY(h, hipStreamWaitEvent(h->ls, h->ev_trained[bi], 0));
  }
  // the rows this batch bypassed were trained on in HBM copies: back to the backing tier,
  // together with the commit of the next batch when that one is waiting
  if (h->deferred >= 0) {
    const int d = h->deferred;
    h->deferred = -1;
    int rc = enqueue_commit(h, d, true);
    return rc ? rc : pump_queue(h);
  }
  {
    // no batch has been prefetched after this one, so no transfer has run since its commit: the
    // overflow copies that commit parked (the previous batch's) go home first, then this batch's
    const BatchBuf &b = h->buf[bi];
    const BatchBuf *parked_prev = (b.parks_prev && b.prev_bi >= 0) ? &h->buf[b.prev_bi] : nullptr;
    HIP_TRY(h, launch_ovf_writeback(b, parked_prev, h->st, h->d_rb, h->d_bytes + 1, h->ls));
    if (h->deep) {  // the marks of these rows go with the next prefetch; the buffer is free once they are home
      HIP_TRY(h, hipEventRecord(h->ev_home[bi], h->ls));
      h->home_recorded[bi] = true;
      h->home_pending[bi] = true;
    }
  }
  return pump_queue(h);
}

int tbe_backward_update(tbe_handle h, const float *d_grad_out, float lr, float eps) {
  if (!h) return TBE_EINVAL;
  return backward_update_with(h, d_grad_out, lr, eps, h->partials);
}

// bytes of partial sums a batch of this handle can need at most
static size_t static_scratch_needed(const tbe_ctx *h) { return 4 * (size_t)h->g.partial_stride * h->huge_slots; }

int tbe_backward_update_static(tbe_handle h, const float *d_grad_out, float lr, float eps) {
  if (!h) return TBE_EINVAL;
  if (h->profiling) return fail(h, TBE_EORDER, "backward_update_static: stage timing is on (it creates events)");
  if (static_scratch_needed(h) > kStaticScratchBytes)
    return fail(h, TBE_ELIMIT, "backward_update_static: a batch of max_lookups could need " +
                                   std::to_string(static_scratch_needed(h)) + " bytes of partial sums, the static scratch holds " +
                                   std::to_string(kStaticScratchBytes));
  int dev = -1;
  HIP_TRY(h, hipGetDevice(&dev));
  if (dev != h->device || !h->static_partials)
    return fail(h, TBE_EORDER, "backward_update_static: the handle was created on another GPU than the current one");
  return backward_update_with(h, d_grad_out, lr, eps, h->static_partials);
}

int tbe_flush(tbe_handle h) {
  if (!h) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  if (h->n_pend > 0 || h->current >= 0 || !h->queued.empty()) {
    // Allowed only after the device has refused a batch (bad offsets, index out of range): that batch and
    // any behind it do nothing and never will (the error sticks), so they are dropped here and the flush
    // brings the backing tier up to the last batch that trained.
    (void)collect_device_errors(h);
    if (!h->sticky) return fail(h, TBE_EORDER, "flush: a batch is still in flight");
    h->n_pend = 0;
    h->current = -1;
    h->deferred = -1;
    h->queued.clear();
  }
  for (int x = 0; x < h->nbuf; x++)  // deep pipeline: bypassed rows that went home after their backward
    if (h->home_pending[x]) {
      HIP_TRY(h, launch_unmark_bypassed(h->buf[x], x, h->st, h->cs));
      h->home_pending[x] = false;
    }
  HIP_TRY(h, launch_transfer(nullptr, h->st, h->l2, h->di, h->throttle, 0, h->d_rb, h->d_bytes, h->d_bytes + 1, h->cs));  // parked victims first
  if (h->prev_buf >= 0) {
    // Every copy in the backing tier is current now, so the next batch must find no row marked
    // "still on its way".  Left in place, such a mark would make that batch ask the transfer to skip
    // a write-back that has already happened, and the request would hit a later batch's victim.
    const BatchBuf &last = h->buf[h->prev_buf];
    HIP_TRY(h, launch_unmark(h->d_tm, last, (last.parks_prev && last.prev_bi >= 0) ? &h->buf[last.prev_bi] : nullptr, h->st,
                             h->l2, h->cs));
    h->prev_buf = -1;
  }
  HIP_TRY(h, launch_flush(h->d_tm, h->g, h->tags, h->l2, h->d_bytes, h->d_bytes + 1, h->cs));  // also slot accumulators -> dev_m
  for (const TableMeta &m : h->tm) {
    HIP_TRY(h, hipMemcpyAsync(m.host_m, m.dev_m, 4 * (size_t)m.rows, hipMemcpyDeviceToHost, h->cs));
    h->flush_state_bytes += 4 * m.rows;
  }
  rc = sync_all(h);
  if (rc) return rc;
  return collect_device_errors(h);
}

int tbe_set_policy(tbe_handle h, int32_t policy) {
  if (!h) return TBE_EINVAL;
  if (policy != TBE_POLICY_LRU && policy != TBE_POLICY_LFU) return fail(h, TBE_EINVAL, "set_policy: unknown policy");
  if (h->k != 0) return fail(h, TBE_EORDER, "set_policy: batches have been prefetched already");
  h->policy = policy;
  return TBE_OK;
}

int tbe_set_backing_throttle(tbe_handle h, int64_t ns_per_row) {
  if (!h) return TBE_EINVAL;
  if (ns_per_row < 0 || ns_per_row > 100000000) return fail(h, TBE_EINVAL, "set_backing_throttle: 0 .. 1e8 ns per row");
  int khz = 0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, h->device) != hipSuccess || khz < 1) khz = 2400000;
  (void)hipGetLastError();
  // one pause is s_sleep 127: about 127 x 64 clocks
  const double clocks = (double)ns_per_row * 1e-9 * (double)khz * 1e3;
  h->throttle.pauses = ns_per_row == 0 ? 0 : std::max(1, (int)(clocks / (127.0 * 64.0) + 0.5));
  return TBE_OK;
}

int tbe_set_probe_grouping(tbe_handle h, int32_t min_windows) {
  if (!h) return TBE_EINVAL;
  if (min_windows < 1 || min_windows > (1 << 30)) return fail(h, TBE_EINVAL, "set_probe_grouping: 1 .. 2^30 windows");
  h->g.probe_min_windows = min_windows;
  return TBE_OK;
}

int tbe_enable_second_level(tbe_handle h, int32_t factor) {
  if (!h) return TBE_EINVAL;
  if (factor < 1 || factor > 1024) return fail(h, TBE_EINVAL, "enable_second_level: factor must be 1..1024");
  if (h->k != 0) return fail(h, TBE_EORDER, "enable_second_level: batches have been prefetched already");
  if (h->l2.on) return fail(h, TBE_EORDER, "enable_second_level: already enabled");
  if (h->deep) return fail(h, TBE_EORDER, "enable_second_level: not together with a prefetch depth above one");
  if (h->st.max_inserts >= (1ll << 29)) return fail(h, TBE_ELIMIT, "enable_second_level: too many possible inserts per batch");
  int64_t slots2 = 0;
  size_t bytes2 = 0;
  for (TableMeta &m : h->tm) {
    if ((int64_t)m.sets * factor * h->g.ways + slots2 >= (1ll << 31)) return fail(h, TBE_ELIMIT, "enable_second_level: too many second-level slots");
    slots2 += (int64_t)m.sets * factor * h->g.ways;
    bytes2 += (size_t)m.sets * factor * h->g.ways * m.row_bytes;
  }
  if (slots2 == 0) return fail(h, TBE_EINVAL, "enable_second_level: no table has a first-level cache");
  HIP_TRY(h, hipHostMalloc((void **)&h->lines2, bytes2, hipHostMallocDefault));
  h->l2.lines_lo = h->lines2;
  h->l2.lines_hi = h->lines2 + bytes2;
  Level2 &l2 = h->l2;
  const size_t M = (size_t)h->st.max_inserts;
  HIP_TRY(h, h->mem.get(&l2.tags2, 4 * (size_t)slots2));
  HIP_TRY(h, h->mem.get(&l2.ts2, 4 * (size_t)slots2));
  HIP_TRY(h, hipMemset(l2.tags2, 0xFF, 4 * (size_t)slots2));
  HIP_TRY(h, hipMemset(l2.ts2, 0xFF, 4 * (size_t)slots2));
  for (int p2 = 0; p2 < 2; p2++) {
    HIP_TRY(h, h->mem.get(&l2.out2[p2], M * h->st.stride));
    // the skip flags of the staged second-level victims follow those of the first-level ones
    HIP_TRY(h, h->mem.get(&h->st.wb_skip[p2], 2 * M));
    HIP_TRY(h, hipMemset(h->st.wb_skip[p2], 0, 2 * M ? 2 * M : 1));
  }
  HIP_TRY(h, h->mem.get(&l2.wb2_dst, 8 * M));
  HIP_TRY(h, hipMemset(l2.wb2_dst, 0, 8 * M ? 8 * M : 8));
  HIP_TRY(h, h->mem.get(&h->d_l2tot, 8 * 4));
  HIP_TRY(h, hipMemset(h->d_l2tot, 0, 8 * 4));
  for (int i = 0; i < h->nbuf; i++) {
    BatchBuf &b = h->buf[i];
    const size_t N = (size_t)std::max<int64_t>(h->max_lookups, 1);
    HIP_TRY(h, h->mem.get(&b.src2, 4 * N));
    HIP_TRY(h, h->mem.get(&b.dst2, 4 * N));
    HIP_TRY(h, h->mem.get(&b.evict2, 4 * N));
    HIP_TRY(h, h->mem.get(&b.ins_dst, 8 * N));
    HIP_TRY(h, h->mem.get(&b.l2v_src, 8 * N));
    HIP_TRY(h, h->mem.get(&b.l2v_dst, 8 * N));
    HIP_TRY(h, h->mem.get(&b.l2v_key, 4 * N));
  }
  int64_t base = 0;
  size_t off = 0;
  for (TableMeta &m : h->tm) {
    m.sets2 = m.sets * (uint32_t)factor;
    m.slot2_base = (int32_t)base;
    m.lines2 = h->lines2 + off;
    base += (int64_t)m.sets2 * h->g.ways;
    off += (size_t)m.sets2 * h->g.ways * m.row_bytes;
  }
  HIP_TRY(h, hipMemcpy(h->d_tm, h->tm.data(), sizeof(TableMeta) * h->tm.size(), hipMemcpyHostToDevice));
  l2.factor = factor;
  l2.total_slots2 = slots2;
  l2.on = true;
  return TBE_OK;
}

int64_t tbe_num_sets2(tbe_handle h, int32_t table) {
  if (!h || table < 0 || table >= h->g.T) return TBE_EINVAL;
  return h->tm[table].sets2;
}

int tbe_export_second_level_state(tbe_handle h, int32_t table, int64_t *h_tags, int32_t *h_ts) {
  if (!h || table < 0 || table >= h->g.T || !h_tags || !h_ts) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  const TableMeta &m = h->tm[table];
  const size_t n = (size_t)m.sets2 * h->g.ways;
  if (n == 0) return TBE_OK;
  std::vector<int32_t> tmp(n);
  HIP_TRY(h, hipMemcpy(tmp.data(), h->l2.tags2 + m.slot2_base, 4 * n, hipMemcpyDeviceToHost));
  for (size_t i = 0; i < n; i++) h_tags[i] = tmp[i];
  HIP_TRY(h, hipMemcpy(h_ts, h->l2.ts2 + m.slot2_base, 4 * n, hipMemcpyDeviceToHost));
  return TBE_OK;
}

int tbe_get_second_level_stats(tbe_handle h, int64_t *h_last4, int64_t *h_total4) {
  if (!h || !h_last4 || !h_total4) return TBE_EINVAL;
  for (int i = 0; i < 4; i++) h_last4[i] = h_total4[i] = 0;
  if (!h->l2.on) return TBE_OK;
  int rc = sync_all(h);
  if (rc) return rc;
  if (h->last_buf >= 0) {
    BatchCounters c;
    HIP_TRY(h, hipMemcpy(&c, h->buf[h->last_buf].cnt, sizeof(c), hipMemcpyDeviceToHost));
    h_last4[0] = c.l2_hits; h_last4[1] = c.l2_demotions; h_last4[2] = c.l2_evictions; h_last4[3] = c.l2_bypasses;
  }
  unsigned long long t[4];
  HIP_TRY(h, hipMemcpy(t, h->d_l2tot, sizeof(t), hipMemcpyDeviceToHost));
  for (int i = 0; i < 4; i++) h_total4[i] = (int64_t)t[i];
  return collect_device_errors(h);
}

int tbe_enable_deferred_init(tbe_handle h, uint64_t seed, float std) {
  if (!h) return TBE_EINVAL;
  if (!(std >= 0.f)) return fail(h, TBE_EINVAL, "enable_deferred_init: std must be >= 0");
  if (h->k != 0) return fail(h, TBE_EORDER, "enable_deferred_init: batches have been prefetched already");
  if (h->di.tm) return fail(h, TBE_EORDER, "enable_deferred_init: already enabled");
  size_t words = 0;
  for (const TableMeta &m : h->tm) words += ((size_t)m.rows + 31) / 32;
  HIP_TRY(h, h->mem.get(&h->init_bits, 4 * words));
  HIP_TRY(h, hipMemset(h->init_bits, 0, 4 * words));
  size_t off = 0;
  for (TableMeta &m : h->tm) {
    m.init_bits = h->init_bits + off;
    off += ((size_t)m.rows + 31) / 32;
  }
  HIP_TRY(h, hipMemcpy(h->d_tm, h->tm.data(), sizeof(TableMeta) * h->tm.size(), hipMemcpyHostToDevice));
  h->di.tm = h->d_tm;
  h->di.seed = seed;
  h->di.std = std;
  return TBE_OK;
}

int tbe_export_initialised(tbe_handle h, int32_t table, uint8_t *h_flags) {
  if (!h || table < 0 || table >= h->g.T || !h_flags) return TBE_EINVAL;
  if (!h->di.tm) return fail(h, TBE_EORDER, "export_initialised: deferred initialisation is not enabled");
  int rc = sync_all(h);
  if (rc) return rc;
  const TableMeta &m = h->tm[table];
  std::vector<uint32_t> w(((size_t)m.rows + 31) / 32);
  HIP_TRY(h, hipMemcpy(w.data(), m.init_bits, 4 * w.size(), hipMemcpyDeviceToHost));
  for (int64_t r = 0; r < m.rows; r++) h_flags[r] = (uint8_t)((w[(size_t)r >> 5] >> (r & 31)) & 1u);
  return TBE_OK;
}

int tbe_set_pooling(tbe_handle h, int32_t pooling) {
  if (!h) return TBE_EINVAL;
  if (pooling != TBE_POOL_SUM && pooling != TBE_POOL_MEAN && pooling != TBE_POOL_MAX)
    return fail(h, TBE_EINVAL, "set_pooling: unknown pooling mode");
  if (h->k != 0) return fail(h, TBE_EORDER, "set_pooling: batches have been prefetched already");
  if (pooling == TBE_POOL_MAX && !h->buf[0].argpos) {  // who supplied each maximum, and the lookups' positions in their bags
    for (int i = 0; i < h->nbuf; i++) {
      HIP_TRY(h, h->mem.get(&h->buf[i].argpos, 4 * (size_t)h->max_batch * (size_t)h->g.sum_dim));
      HIP_TRY(h, h->mem.get(&h->buf[i].sorted_within, 4 * (size_t)std::max<int64_t>(h->max_lookups, 1)));
    }
  }
  h->pooling = pooling;
  return TBE_OK;
}

int tbe_export_argmax(tbe_handle h, int32_t *d_argmax) {
  if (!h || !d_argmax) return TBE_EINVAL;
  if (h->sticky) return h->sticky;
  if (h->pooling != TBE_POOL_MAX) return fail(h, TBE_EORDER, "export_argmax: the pooling mode is not max");
  if (h->current < 0) return fail(h, TBE_EORDER, "export_argmax: no forwarded batch waits for its update");
  const BatchBuf &b = h->buf[h->current];
  HIP_TRY(h, hipMemcpyAsync(d_argmax, b.argpos, 4 * (size_t)b.batch * (size_t)h->g.sum_dim, hipMemcpyDeviceToDevice, h->cs));
  return TBE_OK;
}

int tbe_set_inputs_ready(tbe_handle h, int32_t ready) {
  if (!h) return TBE_EINVAL;
  h->inputs_ready = ready != 0;
  return TBE_OK;
}

int tbe_set_profiling(tbe_handle h, int32_t enable) {
  if (!h) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  drop_profile(h);
  h->profiling = enable == 2 ? 2 : (enable != 0 ? 1 : 0);
  return TBE_OK;
}

int64_t tbe_get_stage_times(tbe_handle h, int32_t stage, int64_t capacity, float *h_ms) {
  if (!h || stage < 0 || stage >= TBE_NUM_STAGES) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  const auto &v = h->prof[stage];
  if (!h_ms) return (int64_t)v.size();
  if (capacity < (int64_t)v.size()) return fail(h, TBE_ELIMIT, "get_stage_times: capacity too small");
  for (size_t i = 0; i < v.size(); i++) HIP_TRY(h, hipEventElapsedTime(&h_ms[i], v[i].first, v[i].second));
  return (int64_t)v.size();
}

int64_t tbe_num_sets(tbe_handle h, int32_t table) {
  if (!h || table < 0 || table >= h->g.T) return TBE_EINVAL;
  return h->tm[table].sets;
}

int tbe_get_stats(tbe_handle h, tbe_stats *out) {
  if (!h || !out) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  memset(out, 0, sizeof(*out));
  BatchCounters tot;
  unsigned long long b64[8];
  HIP_TRY(h, hipMemcpy(&tot, h->d_total, sizeof(tot), hipMemcpyDeviceToHost));
  HIP_TRY(h, hipMemcpy(b64, h->d_bytes, sizeof(b64), hipMemcpyDeviceToHost));
  if (h->last_buf >= 0) {
    BatchCounters c;
    HIP_TRY(h, hipMemcpy(&c, h->buf[h->last_buf].cnt, sizeof(c), hipMemcpyDeviceToHost));
    out->last.lookups = h->buf[h->last_buf].n;
    out->last.uniques = c.n_uniq;
    out->last.hits = (int64_t)c.hits;
    out->last.inserts = c.n_ins;
    out->last.bypasses = c.n_byp;
    out->last.evictions = (int64_t)c.evictions;
    out->last.hit_lookups = (int64_t)c.hit_lookups;
    out->last_long_rows = c.n_heavy;
  }
  out->total.lookups = h->total_lookups;
  out->total.uniques = (int64_t)b64[2];
  out->total.inserts = (int64_t)b64[3];
  out->total.bypasses = (int64_t)b64[4];
  out->total.hits = (int64_t)tot.hits;
  out->total.evictions = (int64_t)tot.evictions;
  out->total.hit_lookups = (int64_t)tot.hit_lookups;
  out->h2d_bytes = (int64_t)b64[0];
  out->d2h_bytes = (int64_t)b64[1] + h->flush_state_bytes;
  out->late_fetches = (int64_t)b64[5];
  out->batch_id = h->k;
  return collect_device_errors(h);
}

int tbe_export_cache_state(tbe_handle h, int32_t table, int64_t *h_tags, int32_t *h_ts) {
  if (!h || table < 0 || table >= h->g.T || !h_tags || !h_ts) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  const TableMeta &m = h->tm[table];
  const size_t n = (size_t)m.sets * h->g.ways;
  if (n == 0) return TBE_OK;
  std::vector<int32_t> tmp(n);
  HIP_TRY(h, hipMemcpy(tmp.data(), h->tags + m.slot_base, 4 * n, hipMemcpyDeviceToHost));
  for (size_t i = 0; i < n; i++) h_tags[i] = tmp[i];
  HIP_TRY(h, hipMemcpy(h_ts, h->ts + m.slot_base, 4 * n, hipMemcpyDeviceToHost));
  return TBE_OK;
}

int tbe_export_cache_freq(tbe_handle h, int32_t table, int32_t *h_freq) {
  if (!h || table < 0 || table >= h->g.T || !h_freq) return TBE_EINVAL;
  int rc = sync_all(h);
  if (rc) return rc;
  const TableMeta &m = h->tm[table];
  const size_t n = (size_t)m.sets * h->g.ways;
  if (n == 0) return TBE_OK;
  HIP_TRY(h, hipMemcpy(h_freq, h->freq + m.slot_base, 4 * n, hipMemcpyDeviceToHost));
  return TBE_OK;
}

int tbe_import_cache_freq(tbe_handle h, int32_t table, const int32_t *h_freq) {
  if (!h || table < 0 || table >= h->g.T || !h_freq) return TBE_EINVAL;
  if (h->n_pend > 0 || h->current >= 0 || !h->queued.empty()) return fail(h, TBE_EORDER, "import_cache_freq: a batch is still in flight");
  int rc = sync_all(h);
  if (rc) return rc;
  const TableMeta &m = h->tm[table];
  const size_t n = (size_t)m.sets * h->g.ways;
  for (size_t i = 0; i < n; i++)
    if (h_freq[i] < 0) return fail(h, TBE_EINVAL, "import_cache_freq: negative count");
  if (n) HIP_TRY(h, hipMemcpy(h->freq + m.slot_base, h_freq, 4 * n, hipMemcpyHostToDevice));
  return TBE_OK;
}

int64_t tbe_export_batch_events(tbe_handle h, int32_t kind, int64_t capacity, int64_t *h_table, int64_t *h_row,
                                int64_t *h_slot, int64_t *h_old) {
  if (!h || kind < 0 || kind > 2) return TBE_EINVAL;
  if (h->last_buf < 0) return 0;
  int rc = sync_all(h);
  if (rc) return rc;
  const BatchBuf &b = h->buf[h->last_buf];
  BatchCounters c;
  HIP_TRY(h, hipMemcpy(&c, b.cnt, sizeof(c), hipMemcpyDeviceToHost));
  if (c.err) return device_error_code(c.err);
  const int64_t count = kind == 0 ? (int64_t)c.hits : kind == 1 ? c.n_ins : c.n_byp;
  if (!h_table || !h_row) return count;
  if (capacity < count) return fail(h, TBE_ELIMIT, "export_batch_events: capacity too small");
  const size_t U = (size_t)c.n_uniq;
  if (U == 0) return 0;
  std::vector<uint32_t> key(U);
  std::vector<uint8_t> st(U);
  std::vector<int32_t> loc(U), old(U);
  HIP_TRY(h, hipMemcpy(key.data(), b.uniq_key, 4 * U, hipMemcpyDeviceToHost));
  HIP_TRY(h, hipMemcpy(st.data(), b.status, U, hipMemcpyDeviceToHost));
  HIP_TRY(h, hipMemcpy(loc.data(), b.loc_u, 4 * U, hipMemcpyDeviceToHost));
  HIP_TRY(h, hipMemcpy(old.data(), b.old_tag, 4 * U, hipMemcpyDeviceToHost));
  const uint8_t want = kind == 0 ? ST_HIT : kind == 1 ? ST_INSERT : ST_BYPASS;
  int64_t n = 0;
  int t = 0;
  for (size_t u = 0; u < U; u++) {
    if (st[u] != want) continue;
    while (t + 1 < h->g.T && h->tm[t + 1].key_base <= key[u]) t++;
    const TableMeta &m = h->tm[t];
    const uint32_t local = key[u] - m.key_base;
    int64_t row = local;
    if (m.sets) {
      const uint32_t s = local / m.rows_per_set;
      row = (int64_t)(local - s * m.rows_per_set) * m.sets + s;
    }
    h_table[n] = t;
    h_row[n] = row;
    if (kind == 1 && h_slot) h_slot[n] = loc[u] - m.slot_base;
    if (kind == 1 && h_old) h_old[n] = old[u];
    n++;
  }
  return n;
}

}  // extern "C"
