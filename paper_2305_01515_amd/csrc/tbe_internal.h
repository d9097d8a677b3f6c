// Internal declarations shared by the HIP translation units of libtbe (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbe {

constexpr int kWave = 64;                 // CDNA wavefront width
constexpr uint32_t kNoSet = 0xFFFFFFFFu;  // global set id of rows of a table without cache
// Backward work classes by the number of lookups a distinct row has in the batch:
//   1            : updated bag by bag (the gradient is the bag's), flagged in the location word
//   2..kLongRun  : one lane group per row, gradient rows gathered per lookup
//   above        : "heavy" rows.  The table's gradient slice is streamed through LDS tile by tile, once per
//                  (chunk of up to heavy_chunk_rows of the table's heavy rows, bag range),
//                  and every lane group adds up, from LDS, the lookups of its rows that fall into the tile;
//                  the partial sums of a row, one per bag range, are added up by the combine kernel.
//                  (Max pooling, whose gradient is masked per lookup, takes these rows one workgroup each.)
constexpr int kLongRun = 64;
constexpr int kHeavyThreads = 1024;       // workgroup of the tile kernel: 1024 / lanes-per-row lane groups
// rows whose sums a lane group keeps in registers (8 fp16 elements per lane need twice the registers of 4 fp32)
__host__ __device__ constexpr int heavy_rows_per_group(int dtype) { return dtype == 0 ? 8 : 6; }
constexpr int kHeavySplit = 2048;          // a heavy row with more lookups is entered into the heavy list in several
constexpr int kHeavyMaxParts = 64;         // parts (at most this many), each taking every parts-th window of G lookups,
                                           // so that no lane group has a hot row's lookups all to itself
// Gradient tile in LDS (wide rows padded by 16 bytes against bank conflicts).  A big tile matters: the lane groups
// of a wavefront run in lockstep, each over its own row's lookups inside the tile, and the more lookups a tile
// holds per row the less their counts differ (benchmark workload, tile kernel: 32 KB 0.145 ms, 64 KB 0.125, 96 KB 0.110).
#ifndef TBE_HEAVY_TILE_BYTES
#define TBE_HEAVY_TILE_BYTES 98304
#endif
constexpr int kHeavyTileBytes = TBE_HEAVY_TILE_BYTES;    // gradient tile in LDS (rows padded by 16 bytes against bank conflicts)
// (chunk, bag range) work items the ranges are chosen for: one workgroup of 1024 threads per CU that is free for
// them (Geometry::heavy_target: all CUs less those the transfer kernel keeps to itself).  Measured on the benchmark workload (32 chunks, 256 CUs; tile kernel + combine alone, ms): 256 items
// 0.110 + 0.024, 512 items 0.124 + 0.039, 1024 items 0.148 + 0.079 -- more ranges mean more partial sums to write
// and to add up; beside the transfer kernel, which holds 48 CUs: 256 items 0.20 (two rounds), 192 items 0.15.
constexpr int kLinkCus = 48;              // workgroups of the transfer kernel: 1024 threads each, a CU each
constexpr int kHeavyMaxRanges = 128;
#ifndef TBE_HEAVY_ROUNDS
#define TBE_HEAVY_ROUNDS 4
#endif
constexpr int kHeavyRounds = TBE_HEAVY_ROUNDS;  // rounds of (chunk, bag range) work items when one round would make them too long

constexpr uint32_t kWhereOverflow = 0x80000000u;  // in the overflow copies of the batch before
constexpr uint32_t kWhereParked = 0x40000000u;    // among the victims the batch before parked
constexpr uint32_t kWhereIndex = 0x3FFFFFFFu;
// With a pipeline several batches deep the overflow copies of more than one batch are alive: the code of such a
// copy also names its batch buffer (bits 26..29; the index is then 26 bits wide).  Zero in the one-deep pipeline.
constexpr int kWhereBufShift = 26;
constexpr uint32_t kWhereBufIndex = (1u << kWhereBufShift) - 1u;
constexpr int kMaxBatchBufs = 16;

// Per-lookup location word (BatchBuf::loc): where the lookup's row is while its batch trains.
constexpr uint32_t kLocOverflow = 0x80000000u;  // index = overflow slot of a bypassed row, else global cache slot
constexpr uint32_t kLocSingle = 0x40000000u;    // the row has exactly one lookup in this batch
constexpr uint32_t kLocIndex = 0x3FFFFFFFu;

enum Status : uint8_t { ST_MISS = 0, ST_HIT = 1, ST_INSERT = 2, ST_BYPASS = 3 };

// Per-table constants, resident in device memory (array of T).
//
// Sort key of (table t, row r): key_base + (r mod S) * rows_per_set + r div S when the table
// has S > 0 sets, key_base + r otherwise.  It is a bijection of (t, r), ascending in
// (table, set, row), so one radix sort groups the lookups by table, set and row at once.
struct TableMeta {
  int64_t rows;
  uint32_t key_base;      // first sort key of this table
  uint32_t rows_per_set;  // ceil(rows / sets); 0 when sets == 0
  uint32_t sets;          // S_t
  uint32_t set_base;      // global id of set 0
  int32_t slot_base;      // global id of slot 0 (= set_base * ways)
  int32_t dim;
  int32_t dtype;          // 0 fp32, 1 fp16
  int32_t col;            // first output column
  int32_t lanes;          // lanes per row: 16 bytes of the row per lane
  uint32_t row_bytes;
  char *lines;            // device: cache lines of this table [sets*ways, row_bytes]
  float *slot_m;          // device: accumulators of the rows in those lines [sets*ways] (while a row is cached its
                          // accumulator lives here, next to 6 MB of its kind, instead of among those of all rows)
  char *host_w;           // pinned host rows [rows, row_bytes]
  float *host_m;          // host accumulators [rows]: read at create, written at flush
  float *dev_m;           // device: row-wise Adagrad accumulators of ALL rows of the table [rows]: current for
                          // the rows that are not in a cache line (commit moves them in and out with the row)
  // second-level cache (Section 5.3): sets2 = l2_factor * sets, so the second-level sets of the
  // rows of first-level set s are s, s + sets, s + 2 sets, ... and belong to that set alone
  uint32_t sets2;         // 0 = no second level for this table
  int32_t slot2_base;     // global id of second-level slot 0 of this table
  char *lines2;           // pinned host: second-level lines [sets2*ways, row_bytes]
  uint32_t *init_bits;    // device: deferred initialisation, one bit per row (1 = the row has a value); null = off
};

// Device-side scalars of one batch (one per batch buffer).
struct BatchCounters {
  int32_t n_uniq;     // distinct (table,row) of the batch
  int32_t n_touched;  // sets with at least one distinct row (+ pseudo sets of cacheless tables)
  int32_t n_ins;
  int32_t n_byp;
  int32_t n_heavy;    // entries of the heavy list (rows with more than kLongRun lookups, a hot row several times)
  int32_t err;        // 1 = bad offsets, 2 = index out of range, 0 = none
  int32_t h_ranges;   // bag ranges the heavy rows' sums are split over in this batch
  int32_t n_mid;      // rows with 2..kLongRun lookups
  unsigned long long hits, evictions, hit_lookups;
  int32_t n_hchunks;  // (table, up to one workgroup's worth of heavy rows) chunks
  // second level: missed rows found there, victims moved down into it, rows it evicted to the
  // lower tier, victims that found no way and went to the lower tier directly
  int32_t l2_hits, l2_demotions, l2_evictions, l2_bypasses;
  // 1 = the sort payload of a lookup is (bag << within_bits) | position inside the bag, which spares
  // the gather of the bag ids after the sort; 0 = a bag is too long for that, the payload is the
  // lookup's position and the bag comes from bag_of_pos
  int32_t packed;
};

// Arrays of one batch; three of these rotate: batch k+1 is prepared while batch k trains, and
// batch k's bypass list and overflow copies are still read by the commit of batch k+1 while
// batch k+2 is already being prepared.
struct BatchBuf {
  // per lookup
  uint32_t *loc;        // [N] location word of every lookup (kLoc* bits), input order
  int32_t *sorted_bag;  // [N] global bag id (t*B + b) of the i-th lookup in sorted order
  int32_t *bag_of_pos;  // [N] global bag id of lookup j (input order); only written when the sort payload
                        //     does not carry the bag (BatchCounters::packed == 0)
  float *inv_len;       // [T * batch] mean pooling: 1 / lookups of the bag (0 for an empty bag)
  bool mean;            // mean pooling instead of sum: forward and backward weigh by inv_len
  bool maxp;            // max pooling: forward records who supplied each maximum, backward sends the gradient there
  int32_t *argpos;      // [batch * sum_dim] max pooling: position inside its bag of the lookup that supplied the
                        //     maximum of each pooled element (-1 for an empty bag); null unless max pooling is set
  int32_t *sorted_within; // [N] max pooling: position inside its bag of the i-th lookup in sorted order
  uint32_t *uid_sorted; // [N] index of the distinct row of the i-th sorted lookup
  // per distinct row (ascending key)
  uint32_t *uniq_key;   // [N]
  int32_t *run_off;     // [N+1] first sorted position of each distinct row; run_off[U] = N
  uint32_t *uniq_sid;   // [N] global set id or kNoSet
  int32_t *uniq_tab;    // [N] table of the distinct row
  int32_t *loc_u;       // [N] global slot id, or -2-j for the j-th bypassed row
  uint8_t *status;      // [N] Status
  int32_t *old_tag;     // [N] for inserts: row that was evicted, -1 if the entry was free
  // second level, per distinct row (null without one):
  int32_t *src2;        // [N] missed row: global second-level slot it was found in, -1 = not there
  int32_t *dst2;        // [N] insert with a victim: second-level slot the victim moves to, -1 = lower tier
  int32_t *evict2;      // [N] ... and the row that slot held (evicted to the lower tier), -1 = it was free
  uint2 *touched;       // [N] (global set id, first distinct row) of every touched set
  int32_t *ins_idx;     // [N] distinct-row indices of the inserts, ascending; per insert also:
  int32_t *ins_tab;     // [N]   its table
  int32_t *ins_slot;    // [N]   the global slot it takes
  int32_t *ins_old;     // [N]   the row evicted from that slot, -1 if it was free
  uint32_t *ins_key;    // [N]   its sort key
  char **ins_src;       // [N]   where its row is fetched from (lower tier or second-level line)
  char **ins_dst;       // [N]   second level only: where its victim goes (second-level line or lower tier)
  char **l2v_src;       // [N]   second level only: line of the row the victim pushes out of the second
                        //       level (null = none), l2v_dst its row in the lower tier, l2v_key its sort key
  char **l2v_dst;
  uint32_t *l2v_key;
  uint32_t *ins_where;  // [N]   0 = fetch it from the backing tier; else a kWhere* code: the backing-tier
                        //       copy is stale, the current value is in HBM (see Staging::where)
  int32_t *byp_idx;     // [N] distinct-row indices of the bypasses, ascending; per bypass also:
  int32_t *byp_tab;     // [N]   its table
  uint32_t *byp_key;    // [N]   its sort key
  char **byp_src;       // [N]   its row in the backing tier
  uint32_t *byp_where;  // [N]   as ins_where
  char *ovf;            // [N * stride] HBM copies of the bypassed rows while their batch trains
  int32_t *mid_idx;     // [N/2 + 1] rows with 2..kLongRun lookups, in the order of the distinct rows (table order)
  int32_t *heavy;       // [N/32 + 1] rows with more lookups, same order, one entry per part of a row (heavy_parts)
  int32_t *heavy_sub;   // [N/32 + 1] per entry: part number | parts << 16
  int32_t *harrive;     // [N/32 + 1] per entry list position of a row's first part: parts whose sums are in (0 between batches)
  uint4 *hchunks;       // [N/kLongRun + T + 1] (table, first position in `heavy`, count, -)
  int32_t *hg_count;    // [2 * (T + 1)] heavy-list entries per table, then the position of each table's first entry
  int32_t *hperm;       // [N/32 + 1] the heavy list's positions, every table's entries ordered by lookups per entry
                        //     (descending, by power of two): lane groups that share a wavefront get rows of like length
  int32_t *hstart;      // [heavy rows * h_ranges] first sorted position of a heavy row in each bag range
  BatchCounters *cnt;   // device
  // host-side description
  const int64_t *d_indices;
  const int64_t *d_offsets;
  int32_t batch;
  int64_t n;
  int32_t k;
  int32_t prev_bi;      // buffer of the batch prefetched before this one, -1 = none
  bool parks_prev;      // this batch's commit parks the overflow copies of the batch before it among its victims
};

// Scratch shared by all batches (only used inside the prefetch stage, which is serial).
struct SortScratch {
  uint32_t *keys[2];
  uint32_t *vals[2];
  uint32_t *hist;          // [256 * max sort blocks] block histograms, then [256] digit totals
  unsigned long long *blk; // [scan blocks + 1] block sums of the compaction passes
  int32_t *wl;             // [kWorklistBlocks * 4] per-workgroup counts of the backward work lists
  unsigned long long *tally;  // [2 * wavefronts of a compaction pass] (evictions, lookups that hit) per wavefront of
  int tally_waves;            //     the last batch's status pass, and how many wavefronts that pass had
};

// Staging between the cache and the host link (one instance; the prefetch stage is serial).
//   in   : rows fetched ahead for the inserts of the batch being prefetched
//   out  : victims of the last two committed batches (by batch id parity): those of the
//          latest wait to be written back; a row evicted by batch k and wanted again by k+1
//          is taken from here instead of making the round trip over the link
struct Staging {
  char *in;            // [max_inserts * stride]
  char *out[2];        // [(max_inserts + max_parked) * stride] each
  char **wb_dst;       // [max_inserts] backing-tier row of each staged victim (null = none)
  uint32_t *wb_rb;     // [max_inserts] row bytes
  uint8_t *wb_skip[2]; // [max_inserts] by parity of the batch that parked the victim: 1 = the next batch
                       // takes the row straight back (from `out`), so it need not travel to the host
  int32_t *wb_n;       // [0] number of parked victim slots, [1] which `out` holds them (device)
  uint32_t *where;     // [key span] per sort key: 0, or where the row's current value is while its
                       // backing-tier copy is stale (kWhereOverflow | j, kWhereParked | i)
  uint32_t stride;     // bytes per staged row (widest row)
  int64_t max_inserts;
  int64_t max_parked;  // room behind the victims for the overflow copies parked with them (0: they are never parked)
};

// Second-level cache: tags and timestamps in HBM, lines in pinned host memory (TableMeta),
// and the staging of the rows it evicts: such a row is read into `out2` by the transfer of
// the batch that pushes it out and written to the lower tier by the next transfer, exactly
// like a first-level victim parked in Staging::out; its map code is kWhereParked | (max_inserts + i).
struct Level2 {
  bool on = false;
  int32_t factor = 0;
  int64_t total_slots2 = 0;
  int32_t *tags2 = nullptr, *ts2 = nullptr;
  char *out2[2] = {nullptr, nullptr};  // [max_inserts * stride] each, by batch parity
  char **wb2_dst = nullptr;            // [max_inserts] lower-tier row of each staged second-level victim
  const char *lines_lo = nullptr, *lines_hi = nullptr;  // address range of the second-level lines (pinned host memory)
};

// Emulation of a slower backing tier, for measurements only: the transfer kernel pauses after every row it
// reads from or writes to the backing tier proper (not the second-level lines).  0 pauses = off.
struct Throttle {
  int32_t pauses = 0;  // s_sleep instructions of the longest kind per backing-tier row
};

struct Geometry {
  int32_t T, ways;
  int32_t sum_dim;
  int32_t key_bits;     // bits of the largest sort key
  int32_t within_bits;  // bits left for the position inside the bag in a packed sort payload (0 = never packed)
  int32_t partial_stride;  // floats per partial-sum slot (widest row, padded to whole lanes)
  int64_t partial_slots;   // slots of the partial-sum buffer (heavy rows x bag ranges of a batch fit in)
  int32_t probe_min_windows = 4096;  // the probe does not group touched sets while that leaves fewer windows than this
  int32_t heavy_target;    // (chunk, bag range) work items the heavy rows' tile kernel should have: the CUs free for it
  uint32_t ovf_stride;     // bytes per overflow / staging slot (widest row)
  uint32_t total_sets;
  int64_t total_slots;
};

// Tables grouped by (storage type, lanes per row); forward and backward are launched once
// per class.  lanes = dim / elements-per-16-bytes rounded up to a power of two.
constexpr int kMaxClasses = 14;
struct ClassInfo {
  int n_classes;
  int cls_dtype[kMaxClasses];
  int cls_lanes[kMaxClasses];
  int cls_count[kMaxClasses];
  const int32_t *cls_tables[kMaxClasses];  // device: table ids of the class
  const int32_t *table_class;              // device: class of every table
};

// ---- launchers (each enqueues on `s` and returns the HIP status of the launch) ----

hipError_t launch_keygen(const TableMeta *tm, const Geometry &g, const BatchBuf &b, uint32_t *keys, uint32_t *vals,
                         hipStream_t s);
hipError_t launch_sort(const Geometry &g, SortScratch &ss, int64_t n, int *result_buf, hipStream_t s);
// lock: batches before the current one whose ways are locked like the current batch's own (0 in the one-deep pipeline)
hipError_t launch_dedup_probe(const TableMeta *tm, const Geometry &g, const BatchBuf &b, SortScratch &ss,
                              const uint32_t *sorted_keys, const uint32_t *sorted_pos, int32_t *tags, int32_t *ts,
                              int32_t *freq, bool lfu, const Level2 &l2, int lock, hipStream_t s);
// write back the staged victims and (b != null) fetch ahead the rows b's batch inserts
// Deferred initialisation on read (Section 5.4.2): a row of the backing tier has no value until it is
// first fetched; the fetch then makes it up instead of reading it.
struct DeferredInit {
  const TableMeta *tm = nullptr;  // device table descriptions (init_bits); null = off
  unsigned long long seed = 0;
  float std = 0.f;
};

hipError_t launch_transfer(const BatchBuf *b, const Staging &st, const Level2 &l2, const DeferredInit &di,
                           const Throttle &th, int k, const uint32_t *rb_of_table,
                           unsigned long long *bytes_h2d, unsigned long long *bytes_d2h, hipStream_t s);
// look up, for the rows cur inserts or bypasses, whether their backing-tier copy is stale
// and where the current value is; then remove prev's entries from the map and enter cur's
// pp: the batch before prev when prev's commit parked pp's overflow copies (their marks go now), else null
hipError_t launch_classify_mark(const TableMeta *tm, const BatchBuf *pp, const BatchBuf *prev, const BatchBuf &cur,
                                const Staging &st, const Level2 &l2, unsigned long long *n_late, hipStream_t s);
// prev_mode: what becomes of prev's overflow copies: kPrevKeep (nothing), kPrevWrite (to the backing tier now),
// kPrevPark (among this batch's parked victims: the next transfer writes them)
constexpr int kPrevKeep = 0, kPrevWrite = 1, kPrevPark = 2;
// deep: the pipeline is several batches deep -- rows whose current value is an overflow copy of a batch that may
// not have trained yet are left to launch_fixup
hipError_t launch_commit(const TableMeta *tm, const BatchBuf &b, const BatchBuf *prev, int prev_mode, const Staging &st,
                         const Level2 &l2, const uint32_t *rb_of_table, unsigned long long *bytes_d2h, bool deep,
                         hipStream_t s);
// ---- pipeline several batches deep (Section 5.7) ----
// The overflow copies of every batch buffer, by buffer number.
struct OverflowCopies {
  const char *of_buf[kMaxBatchBufs];
};
// which of cur's rows are late (as launch_classify_mark), then: prev's victims are home with cur's transfer, prev's
// bypassed rows keep their marks (they go home after prev's backward: launch_unmark_bypassed), cur's rows are
// entered -- its bypassed rows with the number of its buffer
hipError_t launch_classify_mark_deep(const TableMeta *tm, const BatchBuf *prev, const BatchBuf &cur, int cur_buf,
                                     const Staging &st, unsigned long long *n_late, hipStream_t s);
// the marks of b's bypassed rows go, unless a later batch has entered the row again (the write-back that follows
// b's backward is on the link stream in front of every later transfer)
hipError_t launch_unmark_bypassed(const BatchBuf &b, int buf, const Staging &st, hipStream_t s);
// before b's forward, on the compute stream (every earlier batch has trained): the rows of b whose current value
// was an overflow copy of an earlier batch when b's commit ran are copied from there to where b uses them, and
// the accumulators of those it inserted are taken over again
hipError_t launch_fixup(const TableMeta *tm, const BatchBuf &b, const OverflowCopies &oc, const Staging &st,
                        const uint32_t *rb_of_table, unsigned long long *n_copied, hipStream_t s);
// after the batch's backward: its bypassed rows go from their HBM copies to the backing tier
// parked_prev: the batch whose overflow copies b's commit parked and no transfer has written yet (else null)
hipError_t launch_ovf_writeback(const BatchBuf &b, const BatchBuf *parked_prev, const Staging &st,
                                const uint32_t *rb_of_table, unsigned long long *bytes_d2h, hipStream_t s);
hipError_t launch_unmark(const TableMeta *tm, const BatchBuf &last, const BatchBuf *parked_prev, const Staging &st,
                         const Level2 &l2, hipStream_t s);
hipError_t launch_flush(const TableMeta *tm, const Geometry &g, const int32_t *tags, const Level2 &l2,
                        unsigned long long *bytes_h2d, unsigned long long *bytes_d2h, hipStream_t s);
hipError_t launch_forward_classes(const TableMeta *tm, const ClassInfo &ci, const Geometry &g, const BatchBuf &b,
                                  float *out, hipStream_t s);
hipError_t launch_backward_single_classes(const TableMeta *tm, const ClassInfo &ci, const Geometry &g, const BatchBuf &b,
                                          const float *grad_out, float lr, float eps, hipStream_t s);
// which: kBwdHeavy (tile kernel; under max pooling the workgroup-per-row kernel instead), kBwdCombine (sums of the
// tile kernel's partial sums + update; nothing under max pooling), kBwdShort (rows with 2..kLongRun lookups)
constexpr int kBwdHeavy = 0, kBwdCombine = 1, kBwdShort = 2;
hipError_t launch_backward_classes(int which, const TableMeta *tm, const ClassInfo &ci, const Geometry &g,
                                   const BatchBuf &b, const float *grad_out, float *partials, float lr, float eps,
                                   hipStream_t s);

// ---- small device helpers ----

// Bag ranges of the heavy-row backward for a batch with n_hchunks (table, row group) chunks and n_heavy
// heavy rows: enough ranges for about target_items work items, no more than the partial-sum buffer
// (slot_capacity slots of one row each) holds.  A function of the batch alone, so the summation order is
// reproducible.
__host__ __device__ inline int heavy_ranges(int n_hchunks, int n_heavy, long long slot_capacity, int target_items) {
  if (n_hchunks < 1 || n_heavy < 1) return 1;
  long long r = target_items / n_hchunks;  // rounded down: one round of workgroups
  // With many chunks (a model of many tables, or tables with thousands of heavy rows) one round would leave each
  // workgroup a quarter of a batch or more to sweep alone: four rounds of shorter items then, which also evens out
  // what the tables differ in (heterogeneous model: tile kernel 6.5 -> 1.7 ms).
  if (r < kHeavyRounds) r = ((long long)kHeavyRounds * target_items + n_hchunks - 1) / n_hchunks;
  if (r > kHeavyMaxRanges) r = kHeavyMaxRanges;
  if (r > slot_capacity / n_heavy) r = slot_capacity / n_heavy;
  return r < 1 ? 1 : (int)r;
}

// Heavy rows a workgroup of the tile kernel takes at once, and bags per gradient tile, for rows of
// `lanes` lanes of 16 bytes (4 fp32 or 8 fp16 elements each).
__host__ __device__ inline int heavy_chunk_rows(int lanes, int dtype) { return kHeavyThreads / lanes * heavy_rows_per_group(dtype); }
// parts a heavy row of `len` lookups is split into
__host__ __device__ inline int heavy_parts(int len) {
  const int p = (len + kHeavySplit - 1) / kHeavySplit;
  return p < 1 ? 1 : (p > kHeavyMaxParts ? kHeavyMaxParts : p);
}
// first bag of bag range `range` of R over a batch of B bags per table (the ranges are equal to within one bag, so
// that the workgroups of the tile kernel, one per (chunk, range), have equal shares of the lookups)
__host__ __device__ inline int heavy_range_first(int B, int R, int range) { return (int)((long long)B * range / R); }
__host__ __device__ inline int heavy_tile_bags(int lanes, int dtype) {
  return kHeavyTileBytes / (lanes * (dtype == 0 ? 4 : 8) * 4);
}

// Workgroups are handed to the 8 XCDs (each with an L2 of its own) round robin by their
// linear id.  These helpers turn that id into a position in the work so that every XCD
// owns one contiguous eighth of it and walks it front to back: work is ordered by table,
// so a table's rows and its slice of the output gradient are cached in one L2 instead of
// in all eight.  Only the placement changes; any mapping gives the same results.
constexpr int kXcds = 8;
constexpr int kWorklistBlocks = 1024;  // workgroups that build the backward work lists

// position of linear workgroup `id` of `n` when every workgroup is one unit of work
__device__ inline int xcd_block_position(int id, int n) {
  const int q = n / kXcds, rem = n % kXcds, x = id % kXcds;
  return x * q + (x < rem ? x : rem) + id / kXcds;
}

// [first, end) and step of a grid-stride loop over `n` units, `per_block` units per workgroup
// and pass, confined to the XCD's eighth; gridDim.x must be a multiple of kXcds
__device__ inline void xcd_span(int n, int per_block, int &first, int &end, int &step) {
  const int x = blockIdx.x % kXcds, nb = gridDim.x / kXcds;
  const int lo = (int)((int64_t)n * x / kXcds);
  end = (int)((int64_t)n * (x + 1) / kXcds);
  first = lo + (int)(blockIdx.x / kXcds) * per_block;
  step = nb * per_block;
}

// the same for a kernel whose workgroups are numbered `id` of `nblocks` (a multiple of kXcds)
__device__ inline void xcd_span_of(int id, int nblocks, int n, int per_block, int &first, int &end, int &step) {
  const int x = id % kXcds, nb = nblocks / kXcds;
  const int lo = (int)((int64_t)n * x / kXcds);
  end = (int)((int64_t)n * (x + 1) / kXcds);
  first = lo + (id / kXcds) * per_block;
  step = nb * per_block;
}

// table that owns sort key `key`: last t with key_base[t] <= key
__device__ inline int find_table(const TableMeta *tm, int T, uint32_t key) {
  int lo = 0, hi = T - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (tm[mid].key_base <= key) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__device__ inline uint32_t key_of_row(const TableMeta &m, uint32_t row) {
  if (m.sets == 0) return m.key_base + row;
  uint32_t q = row / m.sets;
  return m.key_base + (row - q * m.sets) * m.rows_per_set + q;
}

__device__ inline uint32_t row_of_key(const TableMeta &m, uint32_t key) {
  uint32_t local = key - m.key_base;
  if (m.sets == 0) return local;
  uint32_t s = local / m.rows_per_set;
  return (local - s * m.rows_per_set) * m.sets + s;
}

}  // namespace tbe
