// Pooled embedding-bag forward (Section 2.1.1) and the sparse backward fused with row-wise
// Adagrad (Section 2.1.2, Section 5.9) over cache lines in HBM; rows that bypassed the
// cache are read from / updated in their HBM overflow copies (written back afterwards).
//
// A row is handled by G lanes, 16 bytes of the row per lane (4 fp32 or 8 fp16 elements);
// kernels are instantiated per storage type and G, tables are grouped into such classes.
#include <hip/hip_fp16.h>
#include "tbe_internal.h"

namespace tbe {

template <int DT> struct Elems { static constexpr int n = DT == 0 ? 4 : 8; };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of a row that the backward reads once and writes once: non-temporal accesses, so that
// these lines are the first to leave L2 and the gradient rows, which are re-read once per lookup,
// stay (measured on the benchmark workload: the kernel of the rows with 2..64 lookups 0.22 -> 0.19 ms,
// the single-lookup kernel 0.20 -> 0.185 ms)
__device__ inline uint4 load_once(const char *p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline void store_once(char *p, const uint4 &r) {
  u32x4 v;
  v.x = r.x; v.y = r.y; v.z = r.z; v.w = r.w;
  __builtin_nontemporal_store(v, (u32x4 *)p);
}

// 1.0f that the compiler cannot see through: `acc = fma(widen(h), one, acc)` then stays a fused
// multiply-add with a binary16 operand (one v_fma_mix_f32 per element) instead of being folded
// back into a conversion followed by an addition (two instructions); the product by one is exact,
// so the sum is rounded exactly as before.  Once the repeats of hot rows hit L2, the gathers of
// the forward are bound by the vector ALU's issue rate, not by memory.
__device__ inline float opaque_one() {
  float one = 1.0f;
  asm volatile("" : "+s"(one));
  return one;
}

template <int DT>
__device__ inline void accumulate(float (&acc)[Elems<DT>::n], const uint4 &v, float one) {
  if constexpr (DT == 0) {
    acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y);
    acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
  } else {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      acc[2 * i] = __builtin_fmaf(__half2float(__ushort_as_half((unsigned short)(w[i] & 0xFFFFu))), one, acc[2 * i]);
      acc[2 * i + 1] = __builtin_fmaf(__half2float(__ushort_as_half((unsigned short)(w[i] >> 16))), one, acc[2 * i + 1]);
    }
  }
}

// value of lane N of each row of 16 lanes, in every lane of that row (a DPP move: no LDS traffic)
template <int N>
__device__ inline uint32_t row_bcast(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x150 + N, 0xF, 0xF, true);
}

typedef const __attribute__((address_space(1))) u32x4 *global_u32x4_ptr;
__device__ inline uint4 load_global16(const char *p) {
  const u32x4 v = *(global_u32x4_ptr)(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// N of a chunk's sixteen lookups (Q0 .. Q0+N-1): every lane takes the row's address from the
// lane that computed it and loads its 16 bytes -- all N loads are issued before the first is
// waited for -- then the N are added up in lookup order.
constexpr int kFwdInFlight = 8;  // row loads a lane issues before it waits (4, 8 and 16 measure alike)
template <int DT, int Q0, int N, int X = 0>
__device__ inline void gather_issue(uint4 (&v)[N], uint32_t ptr_lo, uint32_t ptr_hi, int nq, int lig, bool active) {
  if constexpr (X < N) {
    const uint64_t a = ((uint64_t)row_bcast<Q0 + X>(ptr_hi) << 32) | row_bcast<Q0 + X>(ptr_lo);
    if (active && Q0 + X < nq) v[X] = load_global16((const char *)a + lig * 16);
    gather_issue<DT, Q0, N, X + 1>(v, ptr_lo, ptr_hi, nq, lig, active);
  }
}
template <int DT, int Q0, int N>
__device__ inline void gather_rows(float (&acc)[Elems<DT>::n], uint32_t ptr_lo, uint32_t ptr_hi, int nq, int lig,
                                   bool active, float one) {
  uint4 v[N];  // v[x] is loaded and used under the same condition
  gather_issue<DT, Q0, N>(v, ptr_lo, ptr_hi, nq, lig, active);
#pragma unroll
  for (int x = 0; x < N; x++)
    if (active && Q0 + x < nq) accumulate<DT>(acc, v[x], one);
}

// --------------------------------------------------------------------------------------
// forward: one group of G lanes per bag; the bag's locations are read G at a time
// (coalesced) and handed round the group by lane shuffles, four row loads in flight.
// --------------------------------------------------------------------------------------
template <int DT, int G>
__global__ __launch_bounds__(256) void forward_kernel(const TableMeta *__restrict__ tm,
                                                      const int32_t *__restrict__ class_tables, int B, int sum_dim,
                                                      const int64_t *__restrict__ offsets,
                                                      const uint32_t *__restrict__ loc,
                                                      const char *__restrict__ ovf, uint32_t ovf_stride,
                                                      const float *__restrict__ inv_len, float *__restrict__ out,
                                                      const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  constexpr int R = G < 4 ? G : 4;  // row loads in flight per lane
  if (cnt->err) return;
  // bags are table-major: each XCD takes an eighth of the (table, bag block) pairs
  const int vb = xcd_block_position(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
  const int t = class_tables[vb / gridDim.x];
  const TableMeta &m = tm[t];
  const int b = (vb % gridDim.x) * (256 / G) + threadIdx.x / G;
  const int lig = threadIdx.x % G;
  if (b >= B) return;
  const bool active = lig * EPL < m.dim;
  const int64_t lo = offsets[(int64_t)t * B + b], hi = offsets[(int64_t)t * B + b + 1];
  const char *lines = m.lines;
  const uint32_t rb = m.row_bytes;
  const int slot_base = m.slot_base;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; e++) acc[e] = 0.f;
  const float one = opaque_one();
  if constexpr (G == 16) {
    // A group is one DPP row of 16 lanes.  Lane i works out the address of the chunk's i-th
    // lookup once; the sixteen are then visited in four unrolled quartets, each lane fetching
    // the address by a row broadcast (two moves) instead of recomputing it from the location
    // word (a dozen instructions, two of them 64-bit multiplies).
    const int len = (int)(hi - lo);
    for (int c = 0; c < len; c += 16) {
      const int nq = len - c < 16 ? len - c : 16;
      uint64_t my_ptr = 0;
      if (lig < nq) {
        const uint32_t l = loc[lo + c + lig];
        const uint32_t ix = l & kLocIndex;
        my_ptr = (uint64_t)((l & kLocOverflow) ? ovf + (size_t)ix * ovf_stride : lines + (size_t)((int)ix - slot_base) * rb);
      }
      const uint32_t ptr_lo = (uint32_t)my_ptr, ptr_hi = (uint32_t)(my_ptr >> 32);
      constexpr int F = kFwdInFlight;
      gather_rows<DT, 0, F>(acc, ptr_lo, ptr_hi, nq, lig, active, one);
      if constexpr (F < 16)
        if (nq > F) gather_rows<DT, F, F>(acc, ptr_lo, ptr_hi, nq, lig, active, one);
      if constexpr (F < 8) {
        if (nq > 2 * F) gather_rows<DT, 2 * F, F>(acc, ptr_lo, ptr_hi, nq, lig, active, one);
        if (nq > 3 * F) gather_rows<DT, 3 * F, F>(acc, ptr_lo, ptr_hi, nq, lig, active, one);
      }
    }
  } else {
    for (int64_t j0 = lo; j0 < hi; j0 += G) {
      const int nq = (int)((hi - j0) < G ? (hi - j0) : G);
      const uint32_t my_loc = lig < nq ? loc[j0 + lig] : 0u;
      for (int q = 0; q < nq; q += R) {
        uint4 v[R];
#pragma unroll
        for (int x = 0; x < R; x++) {
          const int src = (q + x) & (G - 1);
          const uint32_t l = __shfl(my_loc, src, G);
          const uint32_t ix = l & kLocIndex;
          const char *p = (l & kLocOverflow) ? ovf + (size_t)ix * ovf_stride : lines + (size_t)((int)ix - slot_base) * rb;
          v[x] = (active && q + x < nq) ? *(const uint4 *)(p + lig * 16) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int x = 0; x < R; x++) accumulate<DT>(acc, v[x], one);
      }
    }
  }
  if (inv_len) {  // mean pooling
    const float sc = inv_len[(int64_t)t * B + b];
#pragma unroll
    for (int e = 0; e < EPL; e++) acc[e] *= sc;
  }
  if (active) {
    // written once, read by the model: a non-temporal store, so that the pooled output does not push the
    // tables' hot rows out of L2 (benchmark workload: 0.202 -> 0.197 ms alone, 0.267 -> 0.260 ms beside the other streams)
    float *o = out + (size_t)b * sum_dim + m.col + lig * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      f32x4 v = {acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
      __builtin_nontemporal_store(v, (f32x4 *)(o + e));
    }
  }
}

// Max pooling (Section 2.1.1): element d of the pooled vector is the largest element d among the
// bag's rows; `argpos` records, per pooled element, the position inside the bag of the lookup
// that supplied it -- the first one when several tie (lookups are visited in bag order), -1 for
// an empty bag, whose pooled vector is zero.  The backward sends the gradient there.
template <int DT, int G>
__global__ __launch_bounds__(256) void forward_max_kernel(const TableMeta *__restrict__ tm,
                                                          const int32_t *__restrict__ class_tables, int B, int sum_dim,
                                                          const int64_t *__restrict__ offsets,
                                                          const uint32_t *__restrict__ loc,
                                                          const char *__restrict__ ovf, uint32_t ovf_stride,
                                                          float *__restrict__ out, int32_t *__restrict__ argpos,
                                                          const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  constexpr int R = G < 4 ? G : 4;
  if (cnt->err) return;
  const int vb = xcd_block_position(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
  const int t = class_tables[vb / gridDim.x];
  const TableMeta &m = tm[t];
  const int b = (vb % gridDim.x) * (256 / G) + threadIdx.x / G;
  const int lig = threadIdx.x % G;
  if (b >= B) return;
  const bool active = lig * EPL < m.dim;
  const int64_t lo = offsets[(int64_t)t * B + b], hi = offsets[(int64_t)t * B + b + 1];
  const char *lines = m.lines;
  const uint32_t rb = m.row_bytes;
  const int slot_base = m.slot_base;
  float best[EPL];
  int who[EPL];
#pragma unroll
  for (int e = 0; e < EPL; e++) { best[e] = 0.f; who[e] = -1; }
  for (int64_t j0 = lo; j0 < hi; j0 += G) {
    const int nq = (int)((hi - j0) < G ? (hi - j0) : G);
    const uint32_t my_loc = lig < nq ? loc[j0 + lig] : 0u;
    for (int q = 0; q < nq; q += R) {
      uint4 v[R];
#pragma unroll
      for (int x = 0; x < R; x++) {
        const uint32_t l = __shfl(my_loc, (q + x) & (G - 1), G);
        const uint32_t ix = l & kLocIndex;
        const char *p = (l & kLocOverflow) ? ovf + (size_t)ix * ovf_stride : lines + (size_t)((int)ix - slot_base) * rb;
        v[x] = (active && q + x < nq) ? *(const uint4 *)(p + lig * 16) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int x = 0; x < R; x++) {  // in bag order: a later lookup wins only with a larger value
        if (q + x >= nq) continue;
        float f[EPL];
#pragma unroll
        for (int e = 0; e < EPL; e++) f[e] = 0.f;
        accumulate<DT>(f, v[x], 1.0f);
        const int within = (int)(j0 - lo) + q + x;
#pragma unroll
        for (int e = 0; e < EPL; e++)
          if (who[e] < 0 || f[e] > best[e]) { best[e] = f[e]; who[e] = within; }
      }
    }
  }
  if (active) {
    float *o = out + (size_t)b * sum_dim + m.col + lig * EPL;
    int32_t *a = argpos + (size_t)b * sum_dim + m.col + lig * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      *(float4 *)(o + e) = make_float4(best[e], best[e + 1], best[e + 2], best[e + 3]);
      *(int4 *)(a + e) = make_int4(who[e], who[e + 1], who[e + 2], who[e + 3]);
    }
  }
}

// --------------------------------------------------------------------------------------
// backward
// --------------------------------------------------------------------------------------
template <int DT>
__device__ inline void load_grad(float (&g)[Elems<DT>::n], const float *p) {
#pragma unroll
  for (int e = 0; e < Elems<DT>::n; e += 4) {
    const float4 v = *(const float4 *)(p + e);
    g[e] += v.x; g[e + 1] += v.y; g[e + 2] += v.z; g[e + 3] += v.w;
  }
}

// m += mean(g^2); w -= lr * g / (sqrt(m) + eps), on the 16 bytes this lane owns.
// `sq` is the sum of g^2 over the whole row (already reduced over the group).
template <int DT>
__device__ inline void adagrad_store(char *wp, uint4 raw, const float (&g)[Elems<DT>::n], float m_new, float lr,
                                     float eps);

template <int DT>
__device__ inline void adagrad_apply(char *wp, const float (&g)[Elems<DT>::n], float m_new, float lr, float eps) {
  adagrad_store<DT>(wp, load_once(wp), g, m_new, lr, eps);
}

// the same with the row's 16 bytes already loaded
template <int DT>
__device__ inline void adagrad_store(char *wp, uint4 raw, const float (&g)[Elems<DT>::n], float m_new, float lr,
                                     float eps) {
  // one division per row: the step is w - (lr / (sqrt(m) + eps)) * g, a fused multiply-add per
  // element (an fp32 division costs about a dozen instructions, and the update of the
  // single-lookup rows is bound by the vector ALU otherwise)
  const float step = lr / (sqrtf(m_new) + eps);
  if constexpr (DT == 0) {
    float w[4] = {__uint_as_float(raw.x), __uint_as_float(raw.y), __uint_as_float(raw.z), __uint_as_float(raw.w)};
#pragma unroll
    for (int e = 0; e < 4; e++) w[e] = __builtin_fmaf(-step, g[e], w[e]);
    raw = make_uint4(__float_as_uint(w[0]), __float_as_uint(w[1]), __float_as_uint(w[2]), __float_as_uint(w[3]));
  } else {
    uint32_t wd[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      float a = __half2float(__ushort_as_half((unsigned short)(wd[i] & 0xFFFFu)));
      float b = __half2float(__ushort_as_half((unsigned short)(wd[i] >> 16)));
      a = __builtin_fmaf(-step, g[2 * i], a);
      b = __builtin_fmaf(-step, g[2 * i + 1], b);
      wd[i] = (uint32_t)__half_as_ushort(__float2half_rn(a)) | ((uint32_t)__half_as_ushort(__float2half_rn(b)) << 16);
    }
    raw = make_uint4(wd[0], wd[1], wd[2], wd[3]);
  }
  store_once(wp, raw);
}

struct RowRef {
  char *w;     // the row, where it lives
  float *m;    // its accumulator
};

// The accumulators of all rows stay in HBM (the paper keeps optimizer parameters there,
// Section 5.6.1).  That of a cached row is kept in an array indexed by cache slot (the commit
// moves it there with the row), so the hit path touches a few megabytes of accumulators instead
// of four bytes here and there among those of all rows; a bypassed row's stays where all rows' are.
__device__ inline RowRef locate(const TableMeta &m, uint32_t key, int slot, char *ovf, uint32_t ovf_stride) {
  RowRef r;
  if (slot >= 0) {
    r.w = m.lines + (size_t)(slot - m.slot_base) * m.row_bytes;
    r.m = m.slot_m + (slot - m.slot_base);
  } else {
    r.w = ovf + (size_t)(-2 - slot) * ovf_stride;
    r.m = m.dev_m + row_of_key(m, key);
  }
  return r;
}

// Sum of the output gradients of the lookups [i0, i1) of one row, as seen by one group of G
// lanes: the bag ids are read G at a time (coalesced) and handed round by shuffles, four
// gradient rows are in flight per lane.  `stride_chunks` > 1 lets several groups share a
// range chunk-wise (group `first_chunk` of `stride_chunks`).  Summation order is fixed.
// MODE: kSum, kMean (every gradient row weighs 1 / lookups of its bag, from inv_len) or kMax (a
// lookup receives element d of its bag's gradient only if it supplied the maximum: argbase points
// at the row's columns of the recorded positions, sorted_within gives the lookup's own position).
constexpr int kSum = 0, kMean = 1, kMax = 2;

template <int DT, int G, int MODE>
__device__ inline void reduce_grads(float (&g)[Elems<DT>::n], const float *gbase, const int32_t *sorted_bag, int bag0,
                                    int sum_dim, int i0, int i1, int first_chunk, int stride_chunks, int lig,
                                    bool active, const float *inv_len, const int32_t *argbase,
                                    const int32_t *sorted_within) {
  constexpr int EPL = Elems<DT>::n;
  constexpr bool MEAN = MODE == kMean;
  for (int base = i0 + first_chunk * G; base < i1; base += stride_chunks * G) {
    const int nq = (i1 - base) < G ? (i1 - base) : G;
    const int my_gbag = lig < nq ? sorted_bag[base + lig] : bag0;
    const int my_bag = my_gbag - bag0;
    float my_w = 0.f;  // mean pooling: the weight 1/L of the lookup's bag
    if (MEAN) my_w = lig < nq ? inv_len[my_gbag] : 0.f;
    int my_within = -2;  // max pooling: the lookup's position inside its bag
    if (MODE == kMax) my_within = lig < nq ? sorted_within[base + lig] : -2;
    for (int q = 0; q < nq; q += 4) {
      float4 v[4][EPL / 4];
      float w[4];
#pragma unroll
      for (int x = 0; x < 4; x++) {
        const int bq = __shfl(my_bag, (q + x) & (G - 1), G);
        if (MEAN) w[x] = __shfl(my_w, (q + x) & (G - 1), G);
        int within = 0;
        if (MODE == kMax) within = __shfl(my_within, (q + x) & (G - 1), G);
        const float *p = gbase + (size_t)bq * sum_dim;
        const bool ok = active && (q + x < nq);
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) v[x][e] = ok ? *(const float4 *)(p + 4 * e) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (MODE == kMax && ok) {
          const int32_t *a = argbase + (size_t)bq * sum_dim;
#pragma unroll
          for (int e = 0; e < EPL / 4; e++) {
            const int4 who = *(const int4 *)(a + 4 * e);
            if (who.x != within) v[x][e].x = 0.f;
            if (who.y != within) v[x][e].y = 0.f;
            if (who.z != within) v[x][e].z = 0.f;
            if (who.w != within) v[x][e].w = 0.f;
          }
        }
      }
#pragma unroll
      for (int x = 0; x < 4; x++)
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) {
          if (MEAN) {
            g[4 * e] += v[x][e].x * w[x]; g[4 * e + 1] += v[x][e].y * w[x];
            g[4 * e + 2] += v[x][e].z * w[x]; g[4 * e + 3] += v[x][e].w * w[x];
          } else {
            g[4 * e] += v[x][e].x; g[4 * e + 1] += v[x][e].y; g[4 * e + 2] += v[x][e].z; g[4 * e + 3] += v[x][e].w;
          }
        }
    }
  }
}

// row-wise Adagrad on the row of distinct index u, gradient g spread over the group
template <int DT, int G>
__device__ inline void update_row(const TableMeta &m, uint32_t key, int slot, char *ovf, uint32_t ovf_stride,
                                  const float (&g)[Elems<DT>::n], float lr, float eps, int lig, bool active) {
  constexpr int EPL = Elems<DT>::n;
  float sq = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; e++) sq += g[e] * g[e];
  for (int d = G / 2; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, G);
  const RowRef r = locate(m, key, slot, ovf, ovf_stride);
  const float m_new = *r.m + sq / (float)m.dim;
  if (active) adagrad_apply<DT>(r.w + lig * 16, g, m_new, lr, eps);
  if (lig == 0) *r.m = m_new;
}

// Rows with exactly one lookup in the batch (most distinct rows of a power-law batch):
// their gradient is the bag's gradient, so they are updated bag by bag -- the group holds
// the bag's gradient slice in registers (read once, coalesced) and walks the bag's
// lookups, updating the rows flagged kLocSingle, four rows in flight at a time.  No
// per-lookup gradient read at all.
template <int DT, int G>
__global__ __launch_bounds__(256) void backward_single_kernel(const TableMeta *__restrict__ tm,
                                                              const int32_t *__restrict__ class_tables, int B,
                                                              int sum_dim, const uint32_t *__restrict__ byp_key,
                                                              const int64_t *__restrict__ offsets,
                                                              const uint32_t *__restrict__ loc,
                                                              const float *__restrict__ grad_out, float lr, float eps,
                                                              char *__restrict__ ovf, uint32_t ovf_stride,
                                                              const float *__restrict__ inv_len,
                                                              const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  if (cnt->err) return;
  const int t = class_tables[blockIdx.y];
  const TableMeta &m = tm[t];
  const int b = blockIdx.x * (256 / G) + threadIdx.x / G;
  const int lig = threadIdx.x % G;
  if (b >= B) return;
  const int64_t lo = offsets[(int64_t)t * B + b], hi = offsets[(int64_t)t * B + b + 1];
  if (lo == hi) return;
  const bool active = lig * EPL < m.dim;
  char *lines = m.lines;
  float *slot_m = m.slot_m;
  const uint32_t rb = m.row_bytes;
  const int slot_base = m.slot_base;
  const int gshift = (threadIdx.x & 63) / G * G;  // first lane of this group inside the wavefront
  float g[EPL];
#pragma unroll
  for (int e = 0; e < EPL; e++) g[e] = 0.f;
  if (active) load_grad<DT>(g, grad_out + (size_t)b * sum_dim + m.col + lig * EPL);
  if (inv_len) {  // mean pooling: every lookup of the bag receives 1/L of its gradient
    const float sc = inv_len[(int64_t)t * B + b];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] *= sc;
  }
  float sq = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; e++) sq += g[e] * g[e];
  for (int d = G / 2; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, G);
  const float msq = sq / (float)m.dim;
  for (int64_t j0 = lo; j0 < hi; j0 += G) {
    const int nq = (int)((hi - j0) < G ? (hi - j0) : G);
    const uint32_t my_loc = lig < nq ? loc[j0 + lig] : 0u;
    uint64_t todo = __ballot((my_loc & kLocSingle) != 0) >> gshift;  // the group's single-lookup rows
    if (G < 64) todo &= (1ull << G) - 1ull;
    while (todo) {
      char *w[4];
      float *mp[4];
      float m_old[4];
      uint4 raw[4];
      int n = 0;
#pragma unroll
      for (int x = 0; x < 4; x++) {
        if (todo) {
          const int q = __ffsll((unsigned long long)todo) - 1;
          todo &= todo - 1;
          const uint32_t l = __shfl(my_loc, q, G);
          const uint32_t ix = l & kLocIndex;
          if (l & kLocOverflow) {  // a bypassed row: its copy, and its accumulator among those of all rows
            w[x] = ovf + (size_t)ix * ovf_stride + lig * 16;
            mp[x] = m.dev_m + row_of_key(m, byp_key[ix]);
          } else {
            w[x] = lines + (size_t)((int)ix - slot_base) * rb + lig * 16;
            mp[x] = slot_m + ((int)ix - slot_base);
          }
          m_old[x] = *mp[x];
          if (active) raw[x] = load_once(w[x]);
          n = x + 1;
        }
      }
#pragma unroll
      for (int x = 0; x < 4; x++) {
        if (x < n) {
          const float m_new = m_old[x] + msq;
          if (active) adagrad_store<DT>(w[x], raw[x], g, m_new, lr, eps);
          if (lig == 0) *mp[x] = m_new;
        }
      }
    }
  }
}

// The same for max pooling: the row receives the elements of the bag's gradient whose maximum
// its lookup supplied (recorded by the forward), so the masked gradient and its sum of squares
// differ from row to row.  Rows with exactly one lookup in the batch, bag by bag, the bag's
// gradient slice and the recorded positions of its elements in registers.
template <int DT, int G>
__global__ __launch_bounds__(256) void backward_single_max_kernel(const TableMeta *__restrict__ tm,
                                                              const int32_t *__restrict__ class_tables, int B,
                                                              int sum_dim, const uint32_t *__restrict__ byp_key,
                                                              const int64_t *__restrict__ offsets,
                                                              const uint32_t *__restrict__ loc,
                                                              const float *__restrict__ grad_out, float lr, float eps,
                                                              char *__restrict__ ovf, uint32_t ovf_stride,
                                                              const int32_t *__restrict__ argpos,
                                                              const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  if (cnt->err) return;
  const int t = class_tables[blockIdx.y];
  const TableMeta &m = tm[t];
  const int b = blockIdx.x * (256 / G) + threadIdx.x / G;
  const int lig = threadIdx.x % G;
  if (b >= B) return;
  const int64_t lo = offsets[(int64_t)t * B + b], hi = offsets[(int64_t)t * B + b + 1];
  if (lo == hi) return;
  const bool active = lig * EPL < m.dim;
  char *lines = m.lines;
  float *slot_m = m.slot_m;
  const uint32_t rb = m.row_bytes;
  const int slot_base = m.slot_base;
  const int gshift = (threadIdx.x & 63) / G * G;  // first lane of this group inside the wavefront
  float g[EPL];
#pragma unroll
  for (int e = 0; e < EPL; e++) g[e] = 0.f;
  if (active) load_grad<DT>(g, grad_out + (size_t)b * sum_dim + m.col + lig * EPL);
  int aw[EPL];  // who supplied the maximum of this lane's elements
#pragma unroll
  for (int e = 0; e < EPL; e++) aw[e] = -1;
  if (active) {
    const int32_t *a = argpos + (size_t)b * sum_dim + m.col + lig * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4) {
      const int4 w4 = *(const int4 *)(a + e);
      aw[e] = w4.x; aw[e + 1] = w4.y; aw[e + 2] = w4.z; aw[e + 3] = w4.w;
    }
  }
  const float inv_dim = 1.0f / (float)m.dim;
  for (int64_t j0 = lo; j0 < hi; j0 += G) {
    const int nq = (int)((hi - j0) < G ? (hi - j0) : G);
    const uint32_t my_loc = lig < nq ? loc[j0 + lig] : 0u;
    uint64_t todo = __ballot((my_loc & kLocSingle) != 0) >> gshift;  // the group's single-lookup rows
    if (G < 64) todo &= (1ull << G) - 1ull;
    while (todo) {
      char *w[4];
      float *mp[4];
      float m_old[4];
      uint4 raw[4];
      int within[4];
      int n = 0;
#pragma unroll
      for (int x = 0; x < 4; x++) {
        if (todo) {
          const int q = __ffsll((unsigned long long)todo) - 1;
          todo &= todo - 1;
          const uint32_t l = __shfl(my_loc, q, G);
          const uint32_t ix = l & kLocIndex;
          if (l & kLocOverflow) {  // a bypassed row: its copy, and its accumulator among those of all rows
            w[x] = ovf + (size_t)ix * ovf_stride + lig * 16;
            mp[x] = m.dev_m + row_of_key(m, byp_key[ix]);
          } else {
            w[x] = lines + (size_t)((int)ix - slot_base) * rb + lig * 16;
            mp[x] = slot_m + ((int)ix - slot_base);
          }
          m_old[x] = *mp[x];
          within[x] = (int)(j0 - lo) + q;
          if (active) raw[x] = load_once(w[x]);
          n = x + 1;
        }
      }
#pragma unroll
      for (int x = 0; x < 4; x++) {
        if (x < n) {  // n is the same for all lanes of the group
          float gm[EPL];
          float sq = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; e++) {
            gm[e] = aw[e] == within[x] ? g[e] : 0.f;
            sq += gm[e] * gm[e];
          }
          for (int d = G / 2; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, G);
          const float m_new = m_old[x] + sq * inv_dim;
          if (active) adagrad_store<DT>(w[x], raw[x], gm, m_new, lr, eps);
          if (lig == 0) *mp[x] = m_new;
        }
      }
    }
  }
}

// Rows with 2..kLongRun lookups: one group of G lanes per distinct row, gradients summed
// in sorted (= ascending bag) order.
template <int DT, int G, int MODE>
__global__ __launch_bounds__(256) void backward_short_kernel(const TableMeta *__restrict__ tm, int cls, int B,
                                                             int sum_dim, const int32_t *__restrict__ mid_idx,
                                                             const uint32_t *__restrict__ uniq_key,
                                                             const int32_t *__restrict__ uniq_tab,
                                                             const int32_t *__restrict__ run_off,
                                                             const int32_t *__restrict__ loc_u,
                                                             const int32_t *__restrict__ sorted_bag,
                                                             const float *__restrict__ grad_out, float lr, float eps,
                                                             char *__restrict__ ovf, uint32_t ovf_stride,
                                                             const int32_t *__restrict__ table_class,
                                                             const float *__restrict__ inv_len,
                                                             const int32_t *__restrict__ argpos,
                                                             const int32_t *__restrict__ sorted_within,
                                                             const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  if (cnt->err) return;
  const int n_mid = cnt->n_mid;
  const int lig = threadIdx.x % G;
  int first, end, step;
  xcd_span(n_mid, 256 / G, first, end, step);  // the list is in table order
  for (int i = first + threadIdx.x / G; i < end; i += step) {
    const int u = mid_idx[i];
    const int t = uniq_tab[u];
    if (table_class[t] != cls) continue;
    const int i0 = run_off[u], i1 = run_off[u + 1];
    const TableMeta &m = tm[t];
    const bool active = lig * EPL < m.dim;
    float g[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] = 0.f;
    reduce_grads<DT, G, MODE>(g, grad_out + m.col + lig * EPL, sorted_bag, t * B, sum_dim, i0, i1, 0, 1, lig, active, inv_len,
                              MODE == kMax ? argpos + m.col + lig * EPL : nullptr, sorted_within);
    update_row<DT, G>(m, uniq_key[u], loc_u[u], ovf, ovf_stride, g, lr, eps, lig, active);
  }
}

// Max pooling, and rows narrower than 4 lanes: rows with more than kLongRun lookups, one workgroup per row, its 256/G groups take
// chunks of G lookups round robin; the partial sums are added in group order through LDS.  (The
// gradient a lookup receives is masked by who supplied each maximum, so the bags' gradient rows cannot
// be shared between rows the way the tile kernel below shares them.)
template <int DT, int G, int MODE>
__global__ __launch_bounds__(256) void backward_long_kernel(const TableMeta *__restrict__ tm, int cls, int B,
                                                            int sum_dim, const int32_t *__restrict__ heavy,
                                                            const int32_t *__restrict__ heavy_sub,
                                                            const uint32_t *__restrict__ uniq_key,
                                                            const int32_t *__restrict__ uniq_tab,
                                                            const int32_t *__restrict__ run_off,
                                                            const int32_t *__restrict__ loc_u,
                                                            const int32_t *__restrict__ sorted_bag,
                                                            const float *__restrict__ grad_out, float lr, float eps,
                                                            char *__restrict__ ovf, uint32_t ovf_stride,
                                                            const int32_t *__restrict__ table_class,
                                                            const float *__restrict__ inv_len,
                                                            const int32_t *__restrict__ argpos,
                                                            const int32_t *__restrict__ sorted_within,
                                                            const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  constexpr int NG = 256 / G;
  __shared__ float part[NG][G * EPL + 1];
  if (cnt->err) return;
  const int n_heavy = cnt->n_heavy;
  const int lig = threadIdx.x % G, grp = threadIdx.x / G;
  int first, end, step;
  xcd_span(n_heavy, 1, first, end, step);  // the list is in table order
  for (int it = first; it < end; it += step) {
    if (heavy_sub[it] & 0xFFFF) continue;  // a hot row has several entries: it is taken whole at its first
    const int u = heavy[it];
    const int t = uniq_tab[u];
    if (table_class[t] != cls) continue;  // uniform over the block
    const TableMeta &m = tm[t];
    const bool active = lig * EPL < m.dim;
    float g[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] = 0.f;
    reduce_grads<DT, G, MODE>(g, grad_out + m.col + lig * EPL, sorted_bag, t * B, sum_dim, run_off[u], run_off[u + 1], grp,
                              NG, lig, active, inv_len, MODE == kMax ? argpos + m.col + lig * EPL : nullptr,
                              sorted_within);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < EPL; e++) part[grp][lig * EPL + e] = g[e];
    __syncthreads();
    if (grp == 0) {
#pragma unroll
      for (int e = 0; e < EPL; e++) {
        float s = 0.f;
        for (int q = 0; q < NG; q++) s += part[q][lig * EPL + e];
        g[e] = s;
      }
      update_row<DT, G>(m, uniq_key[u], loc_u[u], ovf, ovf_stride, g, lr, eps, lig, active);
    }
  }
}

// Heavy rows (more than kLongRun lookups; sum and mean pooling).  Such rows carry most of a power-law
// batch's lookups, and the lookups of a row are sorted by bag, so all heavy rows of a table sweep the
// table's slice of the output gradient front to back.  A workgroup takes (table, chunk of the table's
// heavy rows, bag range): it streams the range through LDS tile by tile -- every gradient row is read
// from memory once per chunk, coalesced, the next tile's loads in flight while this one is consumed --
// and each lane group adds up, from LDS, the lookups of its up to kHeavyRowsPerGroup rows that fall
// into the tile (sums in registers).  The partial sums of a row, one per range, go to `partials`; the
// combine kernel adds them in range order and updates the row.
//
// A lane group keeps, per row, a window of G consecutive sorted bag ids (one per lane), how many of
// them it has consumed, and the position of the window; lookups are sorted by bag, so the ones inside
// the tile are a prefix of what is left of the window.
struct HeavySlot {
  int bag;   // this lane's bag id of the window (0x7FFFFFFF outside the row's lookups of this range)
  int next;  // ... of the entry's next window, requested when the one before it is taken up
};
// Beside these, per row of a lane group: `used`, the ids of the window consumed so far (the same in all lanes
// of the group; one byte per row of the group, packed to save vector registers).
struct HeavyState {
  uint64_t used;
};
__device__ inline int heavy_used(const HeavyState &st, int s) { return (int)((st.used >> (8 * s)) & 0xFFu); }
__device__ inline void heavy_set_used(HeavyState &st, int s, int v) {
  st.used = (st.used & ~(0xFFull << (8 * s))) | ((uint64_t)(uint32_t)v << (8 * s));
}

// this lane's bag id of the window that starts at sorted position `at`, for a row whose lookups of the
// range are [lo, hi)
__device__ inline int heavy_window(const int32_t *__restrict__ sorted_bag, int at, int lo, int hi, int lig) {
  const int p = at + lig;
  return (p >= lo && p < hi) ? sorted_bag[p] : 0x7FFFFFFF;
}

// N window positions P0 .. P0+N-1: every lane takes the byte offset of the staged gradient row from the lane
// that holds the lookup and reads its own float4s of that row -- all reads are issued before the first is
// added -- then the N rows are added in lookup order.  A lane's float4s are number lig, G + lig, ... of the
// row, so the lanes of a group read consecutive 16-byte pieces (no two of them in one LDS bank).
template <int DT, int G, int P0, int N, int X = 0>
__device__ inline void heavy_issue(float4 (&v)[N][Elems<DT>::n / 4], const char *tile, uint32_t row_off,
                                   uint32_t lane_off) {
  if constexpr (X < N) {
    const char *src = tile + (row_bcast<P0 + X>(row_off) + lane_off);
#pragma unroll
    for (int e = 0; e < Elems<DT>::n / 4; e++) v[X][e] = *(const float4 *)(src + e * G * 16);
    heavy_issue<DT, G, P0, N, X + 1>(v, tile, row_off, lane_off);
  }
}
template <int DT, int G, int P0, int N>
__device__ inline void heavy_add(float (&g)[Elems<DT>::n], const char *tile, uint32_t row_off, uint32_t lane_off) {
  constexpr int EPL = Elems<DT>::n;
  float4 v[N][EPL / 4];
  heavy_issue<DT, G, P0, N>(v, tile, row_off, lane_off);
#pragma unroll
  for (int x = 0; x < N; x++)
#pragma unroll
    for (int e = 0; e < EPL / 4; e++) {
      g[4 * e] += v[x][e].x; g[4 * e + 1] += v[x][e].y; g[4 * e + 2] += v[x][e].z; g[4 * e + 3] += v[x][e].w;
    }
}

template <int DT, int G, int P0 = 0>
__device__ inline void heavy_add_window(float (&g)[Elems<DT>::n], const char *tile, uint32_t row_off, uint32_t lane_off,
                                        uint64_t positions) {
  constexpr int N = Elems<DT>::n == 8 ? 2 : 4;  // gradient rows read from LDS before they are added
  if constexpr (P0 < G) {
    if (positions & ((uint64_t)((1 << N) - 1) << P0))  // the same for the whole wavefront
      heavy_add<DT, G, P0, N>(g, tile, row_off, lane_off);
    heavy_add_window<DT, G, P0 + N>(g, tile, row_off, lane_off, positions);
  }
}

// win: in LDS, (sorted position of the window after `next`, end of the row's lookups inside this bag range,
// distance between the entry's windows, the entry's position in the heavy list) -- touched once per G lookups,
// so they need not sit in registers
// zero_row: index of a staged row of zeros, read in place of the lookups a group does not have
//
// The lane that holds a lookup of this tile works out the offset of its staged gradient row once; the
// window's positions are then visited in unrolled runs of four, and a run is skipped when no group of the
// wavefront has a lookup of this tile there (a group without one at a position adds the row of zeros).
// Per lookup this costs one DPP addition, the row's LDS reads and its additions (benchmark workload: 27 M vector
// instructions per launch instead of 49 M with the offsets worked out per lookup after a shuffle of the bag id;
// the kernel's time stayed at 0.14 ms: with the additions taken out altogether it takes 0.064 ms, with the
// staging loads taken out 0.12 ms -- what is left is the 3 GB that the lookups read from LDS on the CUs in use).
template <int DT, int G>
__device__ inline uint64_t heavy_consume(HeavySlot &sl, HeavyState &st, int s, int4 *win, float (&g)[Elems<DT>::n], const float *tile,
                                         int row_stride, int zero_row, int base_bag, int end_bag,
                                         const int32_t *__restrict__ sorted_bag, int lig, int gshift) {
  const uint32_t lane_off = (uint32_t)lig * 16u;
  const int group_lane0_x4 = gshift * 4;
  int used = heavy_used(st, s);
  const bool in = lig >= used && sl.bag < end_bag;  // this lane's lookup belongs to the tile and is still to be added
  const uint64_t any = __ballot(in);
  if (any == 0) return 0;
  const uint32_t row_off = (uint32_t)((in ? sl.bag - base_bag : zero_row) * row_stride) * 4u;
  // positions at which some group of the wavefront has a lookup
  uint64_t pos = any;
  if (G <= 32) pos |= pos >> 32;
  if (G <= 16) pos |= pos >> 16;
  if (G <= 8) pos |= pos >> 8;
  if (G <= 4) pos |= pos >> 4;
  if (G < 64) pos &= (1ull << G) - 1ull;
  if constexpr (G == 16) {
    heavy_add_window<DT, G>(g, (const char *)tile, row_off, lane_off, pos);
  } else {  // the same with the positions counted at run time and the offsets permuted through LDS
    constexpr int EPL = Elems<DT>::n;
    constexpr int N = EPL == 8 ? 2 : 4;
#pragma unroll 1
    for (int p = 0; p < G; p += N) {
      if (!((pos >> p) & ((1u << N) - 1u))) continue;  // the same for the whole wavefront
      float4 v[N][EPL / 4];
#pragma unroll
      for (int x = 0; x < N; x++) {
        const uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute(group_lane0_x4 + 4 * (p + x), (int)row_off);
        const char *src = (const char *)tile + (o + lane_off);
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) v[x][e] = *(const float4 *)(src + e * G * 16);
      }
#pragma unroll
      for (int x = 0; x < N; x++)
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) {
          g[4 * e] += v[x][e].x; g[4 * e + 1] += v[x][e].y; g[4 * e + 2] += v[x][e].z; g[4 * e + 3] += v[x][e].w;
        }
    }
  }
  uint64_t mine = any >> gshift;
  if (G < 64) mine &= (1ull << G) - 1ull;
  used += __popcll(mine);  // the group's lanes used .. used + n - 1 held its lookups of this tile
  if (used == G) {         // window used up (else what is left of it lies behind this tile): on to the one requested
    used = 0;              // before, and the one after it is requested now -- it is needed when this one is used up,
    sl.bag = sl.next;      // and the group's other rows are visited in between
    int4 w = *win;
    sl.next = heavy_window(sorted_bag, w.x, 0, w.y, lig);
    w.x += w.z;
    if (lig == 0) *win = w;
  }
  heavy_set_used(st, s, used);
  return any;
}

template <int DT, int G>
__global__ __launch_bounds__(kHeavyThreads) void backward_heavy_kernel(const TableMeta *__restrict__ tm, int cls, int B,
                                                                       int sum_dim, const uint4 *__restrict__ hchunks,
                                                                       const int32_t *__restrict__ heavy,
                                                                       const int32_t *__restrict__ heavy_sub,
                                                                       const int32_t *__restrict__ hperm,
                                                                       const int32_t *__restrict__ hstart,
                                                                       const int32_t *__restrict__ run_off,
                                                                       const int32_t *__restrict__ sorted_bag,
                                                                       const float *__restrict__ grad_out,
                                                                       float *__restrict__ partials, int pstride,
                                                                       const int32_t *__restrict__ table_class,
                                                                       const float *__restrict__ inv_len,
                                                                       const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  constexpr int ROWF = G * EPL;                           // floats per gradient row as the lanes see it
  constexpr int STRIDE = ROWF + (ROWF >= 32 ? 4 : 0);     // ... and per staged row (wide rows: 16 bytes of padding,
                                                          //     so that the groups of a wavefront start in different banks)
  constexpr int TB = kHeavyTileBytes / (ROWF * 4);        // bags per tile (= heavy_tile_bags)
  constexpr int NG = kHeavyThreads / G;                   // lane groups
  constexpr int RPG = heavy_rows_per_group(DT);
  constexpr int PER = kHeavyTileBytes / 16 / kHeavyThreads;  // float4 per thread and tile
  constexpr int PH = PER < 3 ? PER : 3;                      // ... of which this many are requested at a time
  __shared__ float tile[(TB + 1) * STRIDE];  // row TB stays zero
  __shared__ int4 s_win[RPG][NG];  // per (row of a group, group): see heavy_consume
  if (cnt->err) return;
  for (int i = threadIdx.x; i < STRIDE; i += kHeavyThreads) tile[TB * STRIDE + i] = 0.f;
  const int R = cnt->h_ranges;
  const int n_work = cnt->n_hchunks * R;
  const int lig = threadIdx.x % G, grp = threadIdx.x / G;
  const int gshift = (threadIdx.x & 63) / G * G;
  int first, end, step;
  xcd_span(n_work, 1, first, end, step);  // work items are in table order
  for (int wk = first; wk < end; wk += step) {
    const uint4 ch = hchunks[wk / R];  // (table, first position in `heavy`, rows, -)
    const int range = wk % R;
    const int t = (int)ch.x;
    if (table_class[t] != cls) continue;  // uniform over the block
    const TableMeta &m = tm[t];
    const int dim = m.dim, col = m.col;
    const int bag0 = t * B;
    const int range_lo = heavy_range_first(B, R, range), range_hi = heavy_range_first(B, R, range + 1);
    HeavySlot sl[RPG];
    HeavyState st;
    st.used = 0;
    float g[RPG][EPL];
#pragma unroll
    for (int s = 0; s < RPG; s++) {
      const int j = s * NG + grp;  // the chunk's j-th entry in the table's order by length: dealt round the groups
      const bool has = j < (int)ch.z;
      const int h = hperm[(int)ch.y + (has ? j : 0)];
      const int u = heavy[h];
      // The row's lookups of this bag range are the sorted positions [lo, hi).  The row is read in windows of G
      // positions counted from its first lookup; this entry is part `part` of `parts` and takes the windows
      // part, part + parts, ...: the first of them that reaches into the range, its ids before lo counting as used.
      const int sub = heavy_sub[h], part = sub & 0xFFFF, parts = sub >> 16;
      const int run0 = run_off[u];
      const int lo = has ? hstart[h * R + range] : 0;
      const int hi = !has ? 0 : (range + 1 < R ? hstart[h * R + range + 1] : run_off[u + 1]);
      const int w0 = (lo - run0) / G;                               // window that holds position lo
      const int w = w0 + ((part - w0) % parts + parts) % parts;     // first window >= w0 of this part
      const int at = run0 + w * G, stride = parts * G;
      if (lig == 0) s_win[s][grp] = make_int4(at + 2 * stride, hi, stride, has ? h : -1);  // only this group reads it
      heavy_set_used(st, s, (w == w0 && lo > at) ? lo - at : 0);
      sl[s].bag = heavy_window(sorted_bag, at, lo, hi, lig);
      sl[s].next = heavy_window(sorted_bag, at + stride, lo, hi, lig);
#pragma unroll
      for (int e = 0; e < EPL; e++) g[s][e] = 0.f;
    }
    for (int b_first = range_lo; b_first < range_hi; b_first += TB) {  // the range's tiles, TB bags each
      // stage the tile: this thread's share is float4 number k * threads + tid of the tile's TB x ROWF floats,
      // all of them requested before the first is stored
      const int n_f = (min(range_hi, b_first + TB) - b_first) * ROWF;
      __syncthreads();  // the previous tile is no longer read
#pragma unroll
      for (int k0 = 0; k0 < PER; k0 += PH) {  // PH requests in flight, then their stores
        float4 v[PH];
#pragma unroll
        for (int k = 0; k < PH; k++) {
          const int x = ((k0 + k) * kHeavyThreads + threadIdx.x) * 4;
          const int bl = x / ROWF, c = x % ROWF;
          v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (k0 + k < PER && x < n_f && c < dim) {
            v[k] = *(const float4 *)(grad_out + (size_t)(b_first + bl) * sum_dim + col + c);
            if (inv_len) {  // mean pooling: the staged gradient row already carries the bag's 1/L
              const float sc = inv_len[bag0 + b_first + bl];
              v[k].x *= sc; v[k].y *= sc; v[k].z *= sc; v[k].w *= sc;
            }
          }
        }
#pragma unroll
        for (int k = 0; k < PH; k++) {
          const int x = ((k0 + k) * kHeavyThreads + threadIdx.x) * 4;
          if (k0 + k < PER) *(float4 *)(tile + (x / ROWF) * STRIDE + x % ROWF) = v[k];
        }
      }
      __syncthreads();
      const int base_bag = bag0 + b_first, end_bag = bag0 + min(range_hi, b_first + TB);
      // the group's rows are visited in turn, a window's lookups of this tile at a time, until none has any left
      uint64_t busy;
      do {
        busy = 0;
#pragma unroll
        for (int s = 0; s < RPG; s++)
          busy |= heavy_consume<DT, G>(sl[s], st, s, &s_win[s][grp], g[s], tile, STRIDE, TB, base_bag, end_bag, sorted_bag, lig, gshift);
      } while (busy);
    }
    // the sums go to the slots of the groups' heavy-list entries (kept in LDS since the set-up: a load from memory
    // here would wait for the stores in front of it)
#pragma unroll
    for (int s = 0; s < RPG; s++) {
      const int h = s_win[s][grp].w;
      if (h >= 0) {
        // this lane's float4s are number lig, G + lig, ... of the row (see heavy_add)
        float *p = partials + ((size_t)h * R + range) * pstride + lig * 4;
#pragma unroll
        for (int e = 0; e < EPL; e += 4) *(float4 *)(p + e * G) = make_float4(g[s][e], g[s][e + 1], g[s][e + 2], g[s][e + 3]);
      }
    }
  }
}

// Heavy rows: add the partial sums, then update the row.  One lane group per row; the sums of a row's
// parts and bag ranges lie one behind the other and are added in that order (a fixed order, so the result
// is reproducible), four loads in flight.
// sums of one row from which its parts are added up side by side (128: the hot rows of a heterogeneous model pay
// for the fences beside the other streams, its backward 4.6 -> 5.0 ms; 2048: a chain of 2047 sums takes 0.2 ms)
constexpr int kCombineChain = 512;
constexpr int kCombineLoads = 8;  // partial sums a lane group has in flight (4: a chain of 500 sums 0.059 ms, 8: 0.049 ms)
template <int DT, int G>
__global__ __launch_bounds__(256) void backward_combine_kernel(const TableMeta *__restrict__ tm, int cls,
                                                               const int32_t *__restrict__ heavy,
                                                               const int32_t *__restrict__ heavy_sub,
                                                               int32_t *harrive,
                                                               const uint32_t *__restrict__ uniq_key,
                                                               const int32_t *__restrict__ uniq_tab,
                                                               const int32_t *__restrict__ loc_u,
                                                               float *partials, int pstride,
                                                               float lr, float eps, char *__restrict__ ovf,
                                                               uint32_t ovf_stride,
                                                               const int32_t *__restrict__ table_class,
                                                               const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  constexpr int NG = 256 / G;
  if (cnt->err) return;
  const int n_heavy = cnt->n_heavy;
  const int R = cnt->h_ranges;
  const int lig = threadIdx.x % G, grp = threadIdx.x / G;
  int first, end, step;
  xcd_span(n_heavy, NG, first, end, step);  // the list is in table order
  for (int h = first + grp; h < end; h += step) {
    // A row entered once, or a few times, is added up by the lane group of its first entry: parts x R sums in
    // the slots h * R onwards.  For a row with a third of a million lookups that is a chain of 170 parts x 208
    // ranges in one lane group (half a millisecond), so from kCombineChain sums on the work is shared: every part
    // adds up its own R sums, leaves the result in its first slot and counts itself in, and the lane group that
    // finds all the others in adds the parts' sums -- in the order of the parts, whoever it is -- and updates the
    // row.  (The fences this takes write back an XCD's whole L2 each: with them on every row entered twice the
    // benchmark workload's combine took 0.052 instead of 0.019 ms alone and 0.15 instead of 0.03 ms beside the
    // other streams' kernels.  One table, Zipf 1.4, a million lookups: combine 0.53 -> 0.06 ms.)
    const int sub = heavy_sub[h];
    const int part = sub & 0xFFFF, parts = sub >> 16;
    const bool shared = parts > 1 && parts * R >= kCombineChain;
    if (part && !shared) continue;
    const int hf = h - part;
    const int n_sums = shared ? R : parts * R;
    const int u = heavy[h];
    const int t = uniq_tab[u];
    if (table_class[t] != cls) continue;
    const TableMeta &m = tm[t];
    const bool active = lig * EPL < m.dim;
    float g[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] = 0.f;
    float *p0 = partials + (size_t)h * R * pstride + lig * EPL;
    for (int r = 0; r < n_sums; r += kCombineLoads) {
      float4 v[kCombineLoads][EPL / 4];
#pragma unroll
      for (int x = 0; x < kCombineLoads; x++)
#pragma unroll
        for (int e = 0; e < EPL / 4; e++)
          v[x][e] = r + x < n_sums ? *(const float4 *)(p0 + (size_t)(r + x) * pstride + 4 * e) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int x = 0; x < kCombineLoads; x++)
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) {
          g[4 * e] += v[x][e].x; g[4 * e + 1] += v[x][e].y; g[4 * e + 2] += v[x][e].z; g[4 * e + 3] += v[x][e].w;
        }
    }
    if (shared) {
#pragma unroll
      for (int e = 0; e < EPL / 4; e++) *(float4 *)(p0 + 4 * e) = make_float4(g[4 * e], g[4 * e + 1], g[4 * e + 2], g[4 * e + 3]);
      __threadfence();  // the sum is out before this part is counted in
      int before = 0;
      if (lig == 0) before = atomicAdd(harrive + hf, 1);
      before = __shfl(before, 0, G);
      if (before != parts - 1) continue;
      if (lig == 0) harrive[hf] = 0;  // as the next batch expects it
      __threadfence();  // the other parts' sums are read after the count was seen
#pragma unroll
      for (int e = 0; e < EPL; e++) g[e] = 0.f;
      const float *q0 = partials + (size_t)hf * R * pstride + lig * EPL;
      for (int q = 0; q < parts; q++)
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) {
          const float4 v = *(const float4 *)(q0 + (size_t)q * R * pstride + 4 * e);
          g[4 * e] += v.x; g[4 * e + 1] += v.y; g[4 * e + 2] += v.z; g[4 * e + 3] += v.w;
        }
    }
    update_row<DT, G>(m, uniq_key[u], loc_u[u], ovf, ovf_stride, g, lr, eps, lig, active);
  }
}

// --------------------------------------------------------------------------------------
// launchers: one launch per (storage type, G) class present in the model
// --------------------------------------------------------------------------------------
template <int DT, int G>
static void fwd_one(const TableMeta *tm, const int32_t *tables, int count, const Geometry &g, const BatchBuf &b,
                    float *out, hipStream_t s) {
  const int bags_per_block = 256 / G;
  dim3 grid((b.batch + bags_per_block - 1) / bags_per_block, count);
  if (b.maxp)
    hipLaunchKernelGGL((forward_max_kernel<DT, G>), grid, dim3(256), 0, s, tm, tables, b.batch, g.sum_dim, b.d_offsets,
                       b.loc, b.ovf, g.ovf_stride, out, b.argpos, b.cnt);
  else
    hipLaunchKernelGGL((forward_kernel<DT, G>), grid, dim3(256), 0, s, tm, tables, b.batch, g.sum_dim, b.d_offsets,
                       b.loc, b.ovf, g.ovf_stride, b.mean ? b.inv_len : nullptr, out, b.cnt);
}

template <int DT, int G>
static void bwd_one(int which, const TableMeta *tm, int cls, const int32_t *table_class, const Geometry &g,
                    const BatchBuf &b, const float *grad_out, float *partials, float lr, float eps, hipStream_t s) {
  // The tile kernel serves rows of at least 4 lanes (64 bytes); narrower rows, whose lane groups would outnumber
  // what its bookkeeping in LDS is sized for, take the workgroup-per-row kernel, as max pooling does.
  constexpr bool kTiled = G >= 4;
  const bool tiled = kTiled && !b.maxp;
  if (which == kBwdHeavy && tiled) {
    if constexpr (kTiled)
      hipLaunchKernelGGL((backward_heavy_kernel<DT, G>), dim3(1024), dim3(kHeavyThreads), 0, s, tm, cls, b.batch, g.sum_dim,
                         b.hchunks, b.heavy, b.heavy_sub, b.hperm, b.hstart, b.run_off, b.sorted_bag, grad_out, partials, g.partial_stride,
                         table_class, b.mean ? b.inv_len : nullptr, b.cnt);
  } else if (which == kBwdHeavy) {
    auto kern = b.maxp ? backward_long_kernel<DT, G, kMax>
                : b.mean ? backward_long_kernel<DT, G, kMean> : backward_long_kernel<DT, G, kSum>;
    hipLaunchKernelGGL(kern, dim3(8192), dim3(256), 0, s, tm, cls, b.batch, g.sum_dim, b.heavy, b.heavy_sub, b.uniq_key, b.uniq_tab,
                       b.run_off, b.loc_u, b.sorted_bag, grad_out, lr, eps, b.ovf, g.ovf_stride, table_class,
                       b.mean ? b.inv_len : nullptr, b.argpos, b.sorted_within, b.cnt);
  } else if (which == kBwdCombine) {
    if (tiled)
      hipLaunchKernelGGL((backward_combine_kernel<DT, G>), dim3(2048), dim3(256), 0, s, tm, cls, b.heavy, b.heavy_sub, b.harrive,
                         b.uniq_key, b.uniq_tab, b.loc_u, partials, g.partial_stride, lr, eps, b.ovf, g.ovf_stride, table_class,
                         b.cnt);
  } else {
    auto kern = b.maxp ? backward_short_kernel<DT, G, kMax>
                : b.mean ? backward_short_kernel<DT, G, kMean> : backward_short_kernel<DT, G, kSum>;
    hipLaunchKernelGGL(kern, dim3(4096), dim3(256), 0, s, tm, cls, b.batch, g.sum_dim, b.mid_idx, b.uniq_key, b.uniq_tab,
                       b.run_off, b.loc_u, b.sorted_bag, grad_out, lr, eps, b.ovf, g.ovf_stride, table_class,
                       b.mean ? b.inv_len : nullptr, b.argpos, b.sorted_within, b.cnt);
  }
}

template <int DT, int G>
static void bwd_single_one(const TableMeta *tm, const int32_t *tables, int count, const Geometry &g, const BatchBuf &b,
                           const float *grad_out, float lr, float eps, hipStream_t s) {
  const int bags_per_block = 256 / G;
  dim3 grid((b.batch + bags_per_block - 1) / bags_per_block, count);
  if (b.maxp)
    hipLaunchKernelGGL((backward_single_max_kernel<DT, G>), grid, dim3(256), 0, s, tm, tables, b.batch, g.sum_dim,
                       b.byp_key, b.d_offsets, b.loc, grad_out, lr, eps, b.ovf, g.ovf_stride, b.argpos, b.cnt);
  else
    hipLaunchKernelGGL((backward_single_kernel<DT, G>), grid, dim3(256), 0, s, tm, tables, b.batch, g.sum_dim, b.byp_key,
                       b.d_offsets, b.loc, grad_out, lr, eps, b.ovf, g.ovf_stride, b.mean ? b.inv_len : nullptr, b.cnt);
}

#define TBE_DISPATCH(DT, LANES, CALL)                         \
  do {                                                        \
    if ((DT) == 0) {                                          \
      switch (LANES) {                                        \
        case 1: { constexpr int d = 0, l = 1; CALL; } break;  \
        case 2: { constexpr int d = 0, l = 2; CALL; } break;  \
        case 4: { constexpr int d = 0, l = 4; CALL; } break;  \
        case 8: { constexpr int d = 0, l = 8; CALL; } break;  \
        case 16: { constexpr int d = 0, l = 16; CALL; } break;\
        case 32: { constexpr int d = 0, l = 32; CALL; } break;\
        default: { constexpr int d = 0, l = 64; CALL; } break;\
      }                                                       \
    } else {                                                  \
      switch (LANES) {                                        \
        case 1: { constexpr int d = 1, l = 1; CALL; } break;  \
        case 2: { constexpr int d = 1, l = 2; CALL; } break;  \
        case 4: { constexpr int d = 1, l = 4; CALL; } break;  \
        case 8: { constexpr int d = 1, l = 8; CALL; } break;  \
        case 16: { constexpr int d = 1, l = 16; CALL; } break;\
        case 32: { constexpr int d = 1, l = 32; CALL; } break;\
        default: { constexpr int d = 1, l = 64; CALL; } break;\
      }                                                       \
    }                                                         \
  } while (0)

hipError_t launch_forward_classes(const TableMeta *tm, const ClassInfo &ci, const Geometry &g, const BatchBuf &b,
                                  float *out, hipStream_t s) {
  if (b.batch == 0) return hipSuccess;
  for (int c = 0; c < ci.n_classes; c++)
    TBE_DISPATCH(ci.cls_dtype[c], ci.cls_lanes[c], (fwd_one<d, l>(tm, ci.cls_tables[c], ci.cls_count[c], g, b, out, s)));
  return hipGetLastError();
}

hipError_t launch_backward_single_classes(const TableMeta *tm, const ClassInfo &ci, const Geometry &g, const BatchBuf &b,
                                          const float *grad_out, float lr, float eps, hipStream_t s) {
  if (b.n == 0 || b.batch == 0) return hipSuccess;
  for (int c = 0; c < ci.n_classes; c++)
    TBE_DISPATCH(ci.cls_dtype[c], ci.cls_lanes[c],
                 (bwd_single_one<d, l>(tm, ci.cls_tables[c], ci.cls_count[c], g, b, grad_out, lr, eps, s)));
  return hipGetLastError();
}

// A step runs the heavy kernel, the combine, the single-lookup kernel and the short kernel; they
// touch disjoint rows (the combine after the heavy kernel).
hipError_t launch_backward_classes(int which, const TableMeta *tm, const ClassInfo &ci, const Geometry &g,
                                   const BatchBuf &b, const float *grad_out, float *partials, float lr, float eps,
                                   hipStream_t s) {
  if (b.n == 0) return hipSuccess;
  for (int c = 0; c < ci.n_classes; c++)
    TBE_DISPATCH(ci.cls_dtype[c], ci.cls_lanes[c],
                 (bwd_one<d, l>(which, tm, c, ci.table_class, g, b, grad_out, partials, lr, eps, s)));
  return hipGetLastError();
}

}  // namespace tbe
