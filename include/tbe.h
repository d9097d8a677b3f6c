/*
 * tbe.h -- C ABI of the cached embedding-bag training path for AMD MI355X (gfx950).
 *
 * One handle owns a software cache of hot embedding rows in HBM in front of a larger
 * backing tier in pinned host memory, for a set of embedding tables, and runs the
 * per-batch path of DLRM embedding training through it:
 *
 *   prefetch  : decide, for the distinct rows of a batch, hit / insert / bypass, pick the
 *               LRU victims, write the victims back and fetch the missed rows
 *               (paper Section 5.5: tag/state lookup, cache algorithm, data
 *               lookup/update, data movement; Section 5.7: prefetch stage "4a");
 *   forward   : pooled (sum, optionally mean or max) embedding-bag lookup (Section 2.1.1);
 *   backward  : per-row gradient aggregation + row-wise Adagrad applied where the row
 *               lives (Section 2.1.2 Eq. 2, Section 5.9);
 *   flush     : write every cached row back to the backing tier (write-back rule of
 *               Section 5.5.4).
 *
 * Conventions
 *   - every function returns 0 on success or a negative TBE_E* code; no exception
 *     crosses the boundary; tbe_last_error() gives a text for the last failure;
 *   - pointers named d_* are DEVICE pointers, h_* are HOST pointers;
 *   - the caller owns every buffer it passes in; the library owns the cache lines, tags,
 *     timestamps and all scratch memory, allocated once in tbe_create (the optional
 *     second level: in tbe_enable_second_level);
 *   - work is enqueued on the two HIP streams given at creation and the calls return
 *     without waiting for the GPU, except tbe_flush, tbe_get_stats and the tbe_export_*
 *     calls, which synchronise both streams;
 *   - a handle must be driven from one host thread at a time.
 *
 * Cache semantics (deterministic; they define the expected tags and timestamps bit for
 * bit).  Each table t has S_t = cache_slots / ways sets of `ways` entries;
 * row r maps to set r mod S_t.  Batch ids k = 1, 2, ... are assigned by tbe_prefetch.
 * For batch k the distinct rows of each table are handled in two phases (Section 5.5.2
 * lists the steps in this order): 1) every row found in its set is a hit and its entry is
 * stamped k; 2) the remaining rows, in ascending row order, take the entry of their set
 * with the smallest timestamp below k (free entries carry -1; the lowest way wins a
 * tie); the row that was there is evicted and written back, the new row is fetched.  A
 * row whose set has no entry older than k is not cached for this batch ("bypass"): it
 * leaves no trace in tags or timestamps; the library trains it on a temporary HBM copy
 * and writes that back right after the batch's backward.  No row needed by a batch that
 * has not trained is ever evicted (Section 5.7).
 *
 * When the backing tier is current: a row's host copy is stale while the row is cached
 * (write-back cache), while its batch trains if it was bypassed, and while an evicted
 * copy is still on its way; the row-wise accumulators live in HBM for all rows (the paper
 * keeps optimizer parameters there, Section 5.6.1; 4 bytes per row of every table, beside the
 * cache lines) and host_state is only read by tbe_create and written by tbe_flush.  After
 * tbe_flush both host arrays are current.
 *
 * Optional, each selected by one call before the first batch: LFU instead of LRU
 * (tbe_set_policy), mean or max instead of sum pooling (tbe_set_pooling), a second-level cache in
 * pinned host memory between the two tiers (tbe_enable_second_level), initial values made up on
 * first read instead of stored (tbe_enable_deferred_init), a pipeline that fetches several batches
 * ahead (tbe_set_prefetch_depth), a host-side queue of batches in front of tbe_prefetch
 * (tbe_set_prefetch_queue), an emulated slower backing tier for measurements (tbe_set_backing_throttle),
 * one tuning value of the probe (tbe_set_probe_grouping; any time).
 */
#ifndef TBE_H
#define TBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TBE_OK 0
#define TBE_EINVAL (-1)    /* bad argument: null pointer, bad dim / dtype / ways, bad offsets */
#define TBE_ERANGE (-2)    /* an index is outside [0, rows) of its table                      */
#define TBE_EORDER (-3)    /* call order violated (see the functions)                         */
#define TBE_ENOMEM (-4)    /* device or host allocation failed                                */
#define TBE_ELIMIT (-5)    /* batch / lookup count / key space above what create sized        */
#define TBE_EMISMATCH (-6) /* tbe_forward given other buffers than the pending tbe_prefetch   */
#define TBE_EHIP (-7)      /* a HIP runtime call failed                                       */

#define TBE_FP32 0
#define TBE_FP16 1 /* rows stored as IEEE binary16, all arithmetic in fp32, stores round to nearest even */

typedef struct tbe_ctx *tbe_handle;

/* One embedding table (Section 5.2: a two-dimensional tensor in byte-addressable memory). */
typedef struct {
  int64_t rows;        /* H_t >= 1, below 2^31                                                   */
  int32_t dim;         /* D_t: multiple of 4 (fp32) or 8 (fp16), at most 256 (fp32) / 512 (fp16) */
  int32_t dtype;       /* TBE_FP32 or TBE_FP16                                                   */
  void *host_weights;  /* HOST, pinned (hipHostMalloc / tbe_host_alloc), [rows, dim] row-major:  */
                       /* the backing tier; read and written by GPU kernels over the host link   */
  float *host_state;   /* HOST, pinned, [rows]: row-wise Adagrad accumulators; read by tbe_create,  */
                       /* written by tbe_flush (in between they live in HBM)                        */
  int64_t cache_slots; /* HBM slots for this table; S_t = cache_slots / ways (floor); 0 = none   */
} tbe_table_spec;

typedef struct {
  int64_t lookups;     /* N of the batch                                         */
  int64_t uniques;     /* distinct (table, row) pairs                            */
  int64_t hits;        /* distinct rows found in the cache                       */
  int64_t inserts;     /* distinct rows fetched into the cache                   */
  int64_t bypasses;    /* distinct rows not cached for this batch (set overflow) */
  int64_t evictions;   /* rows written back to make room (subset of inserts)     */
  int64_t hit_lookups; /* lookups whose row was a hit (lookup-weighted hit count) */
} tbe_batch_stats;

typedef struct {
  tbe_batch_stats last;  /* last prefetched batch                                   */
  tbe_batch_stats total; /* sum over all batches since create                       */
  int64_t h2d_bytes;     /* backing tier -> cache, since create                       */
  int64_t d2h_bytes;     /* cache -> backing tier (evictions and flushes)           */
  int64_t late_fetches;  /* inserted rows that had to wait for a pending write of   */
                         /* their backing-tier copy (fetched at commit time)        */
  int32_t batch_id;      /* k of the last prefetch                                  */
  int32_t last_long_rows; /* rows of the last batch with more than 64 lookups (segmented backward) */
} tbe_stats;

/*
 * Create a handle (the problem statement of Sections 5.3 and 5.5: a cache class with cache
 * memory, tags and timestamp states per table, managed by GPU kernels).
 *   specs, num_tables : HOST array of table descriptions (copied).
 *   ways              : associativity W, 1..64 (one 64-lane wavefront handles one set).
 *   max_batch         : largest `batch` (samples) of any later call.
 *   max_lookups       : largest `num_lookups` of any later call (at most 2^30).
 *   compute_stream    : hipStream_t on which forward / backward run (NULL = default stream).
 *   aux_stream        : hipStream_t on which prefetch work runs; may equal compute_stream
 *                       (then nothing overlaps).  Both must have the default priority.
 * The sum over tables of the key spans (about the row counts, rounded up to whole sets)
 * must stay below 2^32 (TBE_ELIMIT).  All device memory is allocated here (TBE_ENOMEM): the cache
 * lines and, sized for the worst case of max_lookups distinct rows that all miss, about
 * 5 * max_lookups rows of staging (three batches' copies of bypassed rows, two sets of rows
 * parked for write-back) plus some hundred bytes per lookup of index arrays.
 */
int tbe_create(tbe_handle *out, const tbe_table_spec *specs, int32_t num_tables, int32_t ways,
               int32_t max_batch, int64_t max_lookups, void *compute_stream, void *aux_stream);

/*
 * Prefetch stage (Section 5.7 "4a", Section 5.5.1-5.5.4) for one batch; assigns it the next
 * batch id.
 *   d_indices : DEVICE int64[num_lookups], table-local row ids; the lookups of bag
 *               (t, b) are d_indices[d_offsets[t*batch+b] .. d_offsets[t*batch+b+1]).
 *   d_offsets : DEVICE int64[num_tables*batch + 1], non-decreasing, first 0, last
 *               num_lookups.
 * Both buffers must stay valid and unchanged until the matching tbe_backward_update has
 * completed on the compute stream.  They must have been produced on (or be ordered
 * before) the compute stream at the time of this call.
 * At most ONE batch may be ahead of training: allowed while no more than one batch is
 * prefetched-or-forwarded and not yet updated (else TBE_EORDER).  When such a batch is
 * still in flight, the cache decisions of the new batch are taken as if it had
 * already trained, and the copies that would touch its rows wait for its update.
 * (With tbe_set_prefetch_depth(D), D >= 2: while no more than D batches are prefetched-or-forwarded
 * and not yet updated; the ways of those batches are locked instead, see there.)
 * Bad offsets / out-of-range indices are detected on the device: the batch then does
 * nothing and the error is reported by the next synchronising call (and by later calls).
 */
int tbe_prefetch(tbe_handle h, const int64_t *d_indices, const int64_t *d_offsets, int32_t batch,
                 int64_t num_lookups);

/*
 * Second-level cache (Section 5.3, 5.5.4: two-level exclusive hierarchy).  Adds, between the
 * cache in HBM and the backing tier, a second set-associative LRU cache whose lines the
 * library allocates in pinned host memory: per table factor * S_t sets of `ways` entries,
 * set2(r) = r mod (factor * S_t); tags and timestamps in HBM.  A row lives in exactly one of
 * the three places.  Per batch, after the first level has decided:
 *   (A) every row the first level missed is looked up in the second level: found and inserted
 *       into the first level -> it moves up and its second-level entry becomes free; found but
 *       bypassed by the first level -> it stays, is used in place and is stamped k; not found
 *       -> it comes from / stays in the backing tier;
 *   (B) the rows the first level evicted move down in ascending row order, each into the way
 *       of its second-level set with the smallest timestamp < k - 1 (free first, lowest way
 *       among equals), stamped k; what that way held is written to the backing tier; with no
 *       such way the row goes to the backing tier directly.  Entries stamped by the current
 *       batch or the one before are never replaced (their data may still be in flight).
 * tbe_flush also writes every valid second-level line to the backing tier.  Values do not
 * depend on the hierarchy.  Only before the first tbe_prefetch (TBE_EORDER afterwards or when
 * called twice); allocates (TBE_ENOMEM / TBE_EHIP if that fails); TBE_EINVAL for a factor
 * outside 1..1024 or when no table has a first-level cache; TBE_ELIMIT when 2^31 slots or
 * 2^29 possible inserts per batch are exceeded.
 */
int tbe_enable_second_level(tbe_handle h, int32_t factor);
/* Sets of a table's second-level cache (0 without one). */
int64_t tbe_num_sets2(tbe_handle h, int32_t table);
/* Copy a table's second-level tags and timestamps to HOST arrays of tbe_num_sets2 * ways
 * entries, index set * ways + way.  Synchronises. */
int tbe_export_second_level_state(tbe_handle h, int32_t table, int64_t *h_tags, int32_t *h_ts);
/* Second-level counters of the last prefetched batch and in total, HOST int64[4] each: rows
 * found there, victims moved down into it, rows it evicted to the backing tier, victims
 * that found no way and went to the backing tier directly.  Synchronises. */
int tbe_get_second_level_stats(tbe_handle h, int64_t *h_last4, int64_t *h_total4);

/*
 * Deferred initialisation on read (Section 5.4.2).  With it enabled the rows of the backing
 * tier need no initial values: a row gets its value when it is first fetched from the backing
 * tier (a miss that the second level does not hold) -- normal random numbers std * z made up
 * on the GPU instead of read over the host link, z from a counter-based generator of
 * (seed, table, row, element), so the values do not depend on the order of the reads and equal
 * a table initialised in advance with the same generator:
 *   key   = mix(seed ^ (table + 1) * 0xD1342543DE82EF95),  mix = the finaliser of splitmix64
 *   h_j   = mix(key + row * 0x2545F4914F6CDD1D + element * 3 + j),  j = 0, 1, 2   (64-bit arithmetic)
 *   S     = sum over the twelve 16-bit fields f of h_0, h_1, h_2 of (2 f + 1)  -  12 * 65536
 *   value = fl32( fl32(S) * (std * 2^-17) )     -- z = S / 2^17 is the classic twelve-uniform
 *           approximation of a standard normal number (mean 0, variance 1, |z| < 6)
 * rounded to nearest even when the storage is fp16.  Integer arithmetic and one fp32 product:
 * the stored bits do not depend on who evaluates the definition.  The row reaches host_weights when it is evicted,
 * written back or flushed; rows never read keep whatever host_weights held.  host_state is
 * used as always.  Only before the first tbe_prefetch (TBE_EORDER afterwards or when called
 * twice); allocates one bit per row; TBE_EINVAL for a negative std.
 */
int tbe_enable_deferred_init(tbe_handle h, uint64_t seed, float std);
/* Which rows of a table have a value (1) -- HOST uint8[rows].  Synchronises.  TBE_EORDER when
 * deferred initialisation is not enabled. */
int tbe_export_initialised(tbe_handle h, int32_t table, uint8_t *h_flags);

/*
 * Pooling mode (Section 2.1.1 names sum, mean and max).
 * TBE_POOL_SUM, the default.  TBE_POOL_MEAN: tbe_forward divides every pooled vector by the
 * number of lookups of its bag (a row looked up twice counts twice; an empty bag gives
 * zeros) and tbe_backward_update hands a lookup of a bag of L lookups 1/L of the bag's
 * output gradient.  TBE_POOL_MAX: element d of a pooled vector is the largest element d among
 * the bag's rows (an empty bag gives zeros), and in tbe_backward_update element d of the bag's
 * output gradient goes to the lookup that supplied that maximum -- the first such lookup of
 * the bag when several tie -- and to no other (the first call with TBE_POOL_MAX allocates the
 * record of who supplied each maximum).  Only before the first tbe_prefetch (TBE_EORDER
 * afterwards); TBE_EINVAL for an unknown mode.
 */
#define TBE_POOL_SUM 0
#define TBE_POOL_MEAN 1
#define TBE_POOL_MAX 2
int tbe_set_pooling(tbe_handle h, int32_t pooling);
/*
 * Max pooling (Section 2.1.1): who supplied each maximum of the batch that was forwarded last
 * and has not been updated yet.  d_argmax: DEVICE int32[batch, sum of dims], caller-owned;
 * element [b, col_t + d] = position inside bag (t, b) of the lookup whose row supplied
 * pooled element d (0 = the bag's first lookup; the first of several equal values), -1 for
 * an empty bag.  Written on the compute stream, like tbe_forward's output; does not
 * synchronise.  TBE_EORDER unless the pooling mode is TBE_POOL_MAX and a forwarded batch
 * is waiting for its update.
 */
int tbe_export_argmax(tbe_handle h, int32_t *d_argmax);

/*
 * Replacement policy (Section 5.5.2 names the two that were tried).  TBE_POLICY_LRU, the
 * default: the victim of a miss is the way with the smallest timestamp.  TBE_POLICY_LFU:
 * every entry counts the lookups of its row since it was inserted (a row looked up c times
 * in a batch adds c; saturates at INT32_MAX; forgotten at eviction; free entries count 0)
 * and the victim is the way with the smallest count, the smallest timestamp among equal
 * counts, the lowest way after that.  Everything else -- hits stamped first, misses in
 * ascending row order, ways stamped by the current batch are locked, overflow bypasses --
 * is the same.  The counts are kept under both policies.  Only before the first
 * tbe_prefetch (TBE_EORDER afterwards); TBE_EINVAL for an unknown policy.
 */
#define TBE_POLICY_LRU 0
#define TBE_POLICY_LFU 1
int tbe_set_policy(tbe_handle h, int32_t policy);

/*
 * Prefetch depth (Section 5.7: the caches are accessed several batches in advance, and rows fetched for
 * a batch are not evicted before that batch has trained).  With depth D >= 2 tbe_prefetch may be called
 * for up to D batches beyond the one in training (or about to train), and each of them is fetched into
 * its cache lines right away, beside the training of the batches before it.  The rule of Section 5.7 is a
 * lock: when batch k is decided on, the ways stamped by the batches k - D .. k - 1 -- those that may
 * still wait for their training -- are locked like the ways of batch k itself, so a miss takes the
 * evictable way with the smallest timestamp below k - D (free ways first), and bypasses the cache when
 * the set has none.  Everything else is as at depth 1; pooled outputs and trained values do not depend
 * on the depth, hit, insert and bypass counts do (more rows bypass).  Rows that an earlier batch
 * bypassed and has not written back yet are taken from its copies before the forward of the batch that
 * wants them.  Depth 1 is the default: the next batch is decided on early, but its rows enter their
 * cache lines only after the batch before it has trained, which needs no lock beyond a batch's own.
 * Allocates 2 D - 2 more sets of per-batch buffers (TBE_ENOMEM / TBE_EHIP).  depth 1..7 (TBE_EINVAL);
 * only before the first batch, once, and not together with a second level or a prefetch queue
 * (TBE_EORDER); max_lookups must be below 2^26 (TBE_ELIMIT).  The index buffers of a prefetched batch
 * must stay valid and unchanged until its tbe_backward_update has completed.
 */
int tbe_set_prefetch_depth(tbe_handle h, int32_t depth);
/*
 * The depth in use, and how many rows so far were taken, before a batch's forward, from the copy on which an
 * earlier batch had trained them as bypassed rows (depth >= 2 only; 0 at depth 1).  Synchronises.
 */
int tbe_get_prefetch_depth(tbe_handle h, int32_t *depth, int64_t *rows_from_copies);

/*
 * Queue in front of tbe_prefetch.  With length D > 1 tbe_prefetch accepts up to D batches ahead of
 * training.  This is NOT the multi-batch prefetch of Section 5.7 (that is tbe_set_prefetch_depth):
 * the pipeline itself stays one batch deep, no batch's rows are fetched more than one batch ahead
 * and no lock over several batches exists.  Batches beyond the next one are only kept on the host
 * and their work is issued, in order, as soon as the batch before them has been forwarded.
 * Results are those of a caller that prefetches one batch ahead.  The index buffers of a queued
 * batch must stay valid and unchanged until its tbe_backward_update has completed.  tbe_get_stats and the tbe_export_*
 * calls describe the last batch whose work has been issued, not the last one accepted.
 * length 1..64 (TBE_EINVAL); not while batches are queued and not together with a prefetch depth
 * above one (TBE_EORDER).  Default 1.
 */
int tbe_set_prefetch_queue(tbe_handle h, int32_t length);

/*
 * For measurements, not for production use: emulates a backing tier that is slower than pinned host
 * memory (the paper's lowest tier is storage, Section 5.3).  After every row that the host-link kernel
 * reads from or writes to the backing tier proper -- not the lines of a second-level cache, which stay
 * as fast as they are -- the wavefront that moved it pauses for about ns_per_row nanoseconds (a fixed
 * number of sleep instructions: no wait on memory, so the kernel always ends).  Results do not change,
 * only the time the transfer takes: the backing tier then carries at most about
 * (wavefronts of the kernel, 768) x row bytes / ns_per_row in both directions together.  0 switches it
 * off (the default).
 * Flush, and the write-back that follows a batch without a successor, are not slowed down.
 * May be called at any time between batches; TBE_EINVAL outside 0 .. 1e8.
 */
int tbe_set_backing_throttle(tbe_handle h, int64_t ns_per_row);

/*
 * Tuning of the probe of Section 5.5.1 (results never depend on it): a wavefront of the probe kernel
 * takes several consecutive touched sets at a time when a batch leaves only a few distinct rows per
 * set, but not while that would leave fewer than min_windows wavefronts' worth of work.  Default 4096;
 * 1 groups whenever the rows per set allow it (how the tests reach the grouped path with small
 * models), a huge value never groups.  Any time between batches; TBE_EINVAL outside 1 .. 2^30.
 */
int tbe_set_probe_grouping(tbe_handle h, int32_t min_windows);

/*
 * By default tbe_prefetch orders its work behind everything enqueued on the compute stream
 * so far, because the index buffers may have been produced there.  With ready = 1 the
 * caller guarantees instead that the buffers passed to tbe_prefetch are complete in device
 * memory when the call is made (e.g. a data loader finished them earlier); the prefetch
 * stage of the next batch can then start while the current batch is still training
 * (Section 5.7: the stages of different batches run simultaneously); it is ordered only
 * behind the last tbe_forward launched, whose output the model is waiting for.
 */
int tbe_set_inputs_ready(tbe_handle h, int32_t ready);

/*
 * Pooled lookup (Section 2.1.1, sum pooling): for every table t, sample b and d < D_t
 *   d_out[b * sum_dim + col_t + d] = sum over the bag's lookups j of W_t[d_indices[j]][d]
 * with col_t the sum of the dims of the tables before t; an empty bag gives zeros; fp32
 * accumulation.  d_out: DEVICE float[batch * sum_dim].
 * Consumes the oldest prefetched batch, which must have been prefetched with these same
 * buffers (TBE_EMISMATCH); when nothing is pending it runs the prefetch stage itself
 * first.  TBE_EORDER if the previous forwarded batch has not been updated yet.
 */
int tbe_forward(tbe_handle h, const int64_t *d_indices, const int64_t *d_offsets, int32_t batch,
                int64_t num_lookups, float *d_out);

/*
 * Sparse backward fused with row-wise Adagrad (Section 2.1.2, Section 5.9) for the batch
 * last forwarded: for every distinct row r of table t in it
 *   g[d]  = sum over its lookups j of d_grad_out[bag(j) * sum_dim + col_t + d]
 *   m_r  += (1 / D_t) * sum_d g[d]^2
 *   w_r[d] -= lr * g[d] / (sqrt(m_r) + eps)           (with the new m_r)
 * applied in place to the cache line (or to the temporary copy of a bypassed row).
 * d_grad_out: DEVICE float[batch * sum_dim], ready on the compute stream.
 * TBE_EORDER without a forwarded batch.
 */
int tbe_backward_update(tbe_handle h, const float *d_grad_out, float lr, float eps);

/*
 * tbe_backward_update for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same backward, same kernels, same results, but the one
 * scratch buffer the backward's kernels use -- the partial sums of the rows with the most lookups,
 * which tbe_backward_update keeps in memory that tbe_create allocated -- lies in a fixed array of
 * TBE_STATIC_SCRATCH_BYTES bytes inside the library's device image instead (every GPU the library
 * runs on holds one such array until the process ends).  The call allocates nothing: no hipMalloc,
 * no hipFree, no event or stream creation; it only enqueues kernels and records / waits for events
 * that tbe_create made.
 *   - TBE_ELIMIT when the handle's worst case does not fit: 4 bytes x the widest row's elements (rounded
 *     up to whole 16-byte lanes, a power of two of them) x max(4 * (max_lookups / 65 + 1), 32768) partial
 *     sums above TBE_STATIC_SCRATCH_BYTES -- e.g. dim 128 and max_lookups up to about a million fit; the
 *     error text gives the figure;
 *   - TBE_EORDER while stage timing is on (tbe_set_profiling creates events per call), when the
 *     current GPU is not the one the handle was created on, or without a forwarded batch;
 *   - the array keeps the last call's contents; nothing in it has to start at zero (every partial sum
 *     a batch reads it has written before, in the same call);
 *   - all handles on one GPU share that GPU's array: calls of this function that overlap on one GPU
 *     (two handles whose compute streams run concurrently) race.  tbe_backward_update is not affected.
 * May be mixed freely with tbe_backward_update on the same handle.
 */
#define TBE_STATIC_SCRATCH_BYTES (32u << 20)
int tbe_backward_update_static(tbe_handle h, const float *d_grad_out, float lr, float eps);

/*
 * Write every valid cache line and its accumulator to the backing tier (Section 5.5.4,
 * write-back) and wait for both streams: afterwards the host arrays hold the current model.
 * Tags and timestamps stay.  TBE_EORDER while a batch is prefetched or forwarded but not
 * updated.  Also reports errors the device found earlier: once the device has refused a batch
 * (TBE_EINVAL / TBE_ERANGE, which stick), tbe_flush drops that batch and any behind it, writes
 * the state of the last batch that trained to the backing tier and returns the error code.
 */
int tbe_flush(tbe_handle h);

/* Waits for outstanding work and releases everything the library allocated. */
int tbe_destroy(tbe_handle h);

/* Counters (synchronises).  Hit rate per distinct row = hits / uniques; per lookup =
 * hit_lookups / lookups; requests reaching the backing tier = (1 - hit rate) * requests
 * (Section 4.2, Eq. 4 with alpha the miss ratio). */
int tbe_get_stats(tbe_handle h, tbe_stats *out);

/*
 * Stage timing for measurement (not described by the paper).  While enabled, every call
 * brackets the kernels of each stage with HIP timing events on the stream they are
 * launched on; tbe_get_stage_times returns the elapsed milliseconds of every bracket
 * recorded since profiling was switched on, in call order (at most 16384 per stage).
 * enable = 2 leaves out the brackets of the backward's single kernels (3, 4, 6, 7), which lie inside bracket 8
 * and lengthen it by their own events.  Both calls synchronise; tbe_set_profiling discards earlier records.
 * With h_ms NULL, tbe_get_stage_times returns the number of records.
 */
#define TBE_STAGE_PREFETCH 0       /* key generation, sort, dedup, probe, compaction (aux stream) */
#define TBE_STAGE_FILL 1           /* host link: write-back of parked victims + fetch-ahead of missed rows (aux) */
#define TBE_STAGE_FORWARD 2        /* pooled lookup (compute stream)                              */
#define TBE_STAGE_BACKWARD_COMBINE 3 /* heavy rows: sum of the partial sums + update (compute stream) */
#define TBE_STAGE_BACKWARD_SHORT 4 /* backward of rows with 2..64 lookups (compute stream)          */
#define TBE_STAGE_COMMIT 5         /* victims -> staging, fetched rows -> cache lines (aux stream)  */
#define TBE_STAGE_BACKWARD_SINGLE 6 /* backward of rows with one lookup, bag by bag (compute stream) */
#define TBE_STAGE_BACKWARD_HEAVY 7 /* rows with more than 64 lookups: partial sums per bag range from gradient tiles in LDS
                                      (max pooling: one workgroup per row, update included) (compute stream) */
#define TBE_STAGE_BACKWARD 8       /* the whole backward: from before its first kernel to after its last (compute stream);
                                      brackets 7, 3, 6, 4 lie inside it, one behind the other */
#define TBE_NUM_STAGES 9
int tbe_set_profiling(tbe_handle h, int32_t enable);
int64_t tbe_get_stage_times(tbe_handle h, int32_t stage, int64_t capacity, float *h_ms);

/* Sets and slots of a table's cache: S_t (and S_t * ways slots). */
int64_t tbe_num_sets(tbe_handle h, int32_t table);

/* Copy a table's tags (row id, -1 = free) and timestamps (batch id, -1 = free) to
 * HOST arrays of S_t * ways entries, index set * ways + way.  Synchronises. */
int tbe_export_cache_state(tbe_handle h, int32_t table, int64_t *h_tags, int32_t *h_ts);

/* Copy a table's per-entry lookup counts (see tbe_set_policy; 0 = free) to a HOST array of
 * S_t * ways entries, same order as the tags.  Synchronises. */
int tbe_export_cache_freq(tbe_handle h, int32_t table, int32_t *h_freq);
/* The reverse: overwrite a table's per-entry lookup counts from a HOST array in the same order (values >= 0;
 * restoring a saved cache state, and how the tests reach counts near INT32_MAX).  Synchronises.
 * TBE_EORDER while a batch is prefetched or forwarded but not updated. */
int tbe_import_cache_freq(tbe_handle h, int32_t table, const int32_t *h_freq);

/*
 * Events of the last prefetched batch.  kind 0 = hits, 1 = inserts, 2 = bypasses.
 * Returns the number of events (or a negative error).  With non-null HOST arrays (each at
 * least `capacity` long) fills h_table / h_row, and for inserts h_slot (table-local,
 * set * ways + way) and h_old (row evicted from that slot, -1 if it was free); h_slot and
 * h_old may be null.  Order: ascending (table, set, row).  Synchronises.
 */
int64_t tbe_export_batch_events(tbe_handle h, int32_t kind, int64_t capacity, int64_t *h_table,
                                int64_t *h_row, int64_t *h_slot, int64_t *h_old);

/* Text describing the last error on this handle (static storage; h may be NULL for
 * errors of tbe_create). */
const char *tbe_last_error(tbe_handle h);

/* Pinned, device-visible host memory for the backing tier (existing memory cannot be
 * registered after the fact on every system).  Contents are uninitialised. */
int tbe_host_alloc(void **h_ptr, size_t bytes);
int tbe_host_free(void *h_ptr);

/*
 * Embedding table assignment (Section 5.6.1, Eq. 6), one GPU.  Host function: HOST pointers
 * only, no handle, no GPU work.  Every table is assigned to exactly one memory type such
 * that the tables of a memory type fit its capacity and
 *     time = sum over tables t of traffic_t / bandwidth_{memory of t}
 * is minimal.  traffic = D * L * p of Eq. 6 (bytes the table moves per step, any common
 * unit), bytes = the table's size.  Exact (branch and bound) unless the search visits more
 * than max_nodes nodes (<= 0: 5 million); then the best assignment found so far is returned
 * and *h_optimal is 0.  Outputs: h_memory_of_table[num_tables] (index into mems), *h_time
 * (Eq. 6 of that assignment), *h_optimal; the last two may be null.
 * Errors: TBE_EINVAL (null pointer, no table or memory type, negative size or traffic,
 * bandwidth not positive), TBE_ELIMIT (no assignment fits).
 */
typedef struct {
  int64_t bytes;
  double traffic;
} tbe_place_table;
typedef struct {
  int64_t capacity_bytes;
  double bandwidth;
} tbe_place_memory;
int tbe_plan_placement(const tbe_place_table *tables, int32_t num_tables, const tbe_place_memory *mems,
                       int32_t num_mems, int64_t max_nodes, int32_t *h_memory_of_table, double *h_time,
                       int32_t *h_optimal);

#ifdef __cplusplus
}
#endif
#endif /* TBE_H */
