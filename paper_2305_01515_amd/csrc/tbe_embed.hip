// Pooled embedding-bag forward (Section 2.1.1) and the sparse backward fused with row-wise
// Adagrad (Section 2.1.2, Section 5.9) over cache lines in HBM; rows that bypassed the
// cache are read from / updated in the pinned backing tier directly.
//
// A row is handled by G lanes, 16 bytes of the row per lane (4 fp32 or 8 fp16 elements);
// kernels are instantiated per storage type and G, tables are grouped into such classes.
#include <hip/hip_fp16.h>
#include "tbe_internal.h"

namespace tbe {

template <int DT> struct Elems { static constexpr int n = DT == 0 ? 4 : 8; };

template <int DT>
__device__ inline void accumulate(float (&acc)[Elems<DT>::n], const uint4 &v) {
  if constexpr (DT == 0) {
    acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y);
    acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
  } else {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      acc[2 * i] += __half2float(__ushort_as_half((unsigned short)(w[i] & 0xFFFFu)));
      acc[2 * i + 1] += __half2float(__ushort_as_half((unsigned short)(w[i] >> 16)));
    }
  }
}

// --------------------------------------------------------------------------------------
// forward: one group of G lanes per bag; the bag's locations are read G at a time
// (coalesced) and handed round the group by lane shuffles, four row loads in flight.
// --------------------------------------------------------------------------------------
template <int DT, int G>
__global__ __launch_bounds__(256) void forward_kernel(const TableMeta *__restrict__ tm,
                                                      const int32_t *__restrict__ class_tables, int B, int sum_dim,
                                                      const int64_t *__restrict__ offsets,
                                                      const int32_t *__restrict__ loc,
                                                      const char *__restrict__ ovf, uint32_t ovf_stride,
                                                      float *__restrict__ out, const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  if (cnt->err) return;
  const int t = class_tables[blockIdx.y];
  const TableMeta &m = tm[t];
  const int b = blockIdx.x * (256 / G) + threadIdx.x / G;
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
  for (int64_t j0 = lo; j0 < hi; j0 += G) {
    const int nq = (int)((hi - j0) < G ? (hi - j0) : G);
    const int my_loc = lig < nq ? loc[j0 + lig] : 0;
    for (int q = 0; q < nq; q += 4) {
      uint4 v[4];
#pragma unroll
      for (int x = 0; x < 4; x++) {
        const int src = (q + x) & (G - 1);
        const int l = __shfl(my_loc, src, G);
        const char *p = l >= 0 ? lines + (size_t)(l - slot_base) * rb : ovf + (size_t)(-2 - l) * ovf_stride;
        v[x] = (active && q + x < nq) ? *(const uint4 *)(p + lig * 16) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int x = 0; x < 4; x++) accumulate<DT>(acc, v[x]);
    }
  }
  if (active) {
    float *o = out + (size_t)b * sum_dim + m.col + lig * EPL;
#pragma unroll
    for (int e = 0; e < EPL; e += 4) *(float4 *)(o + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
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
__device__ inline void adagrad_apply(char *wp, const float (&g)[Elems<DT>::n], float m_new, float lr, float eps) {
  const float denom = sqrtf(m_new) + eps;
  uint4 raw = *(const uint4 *)wp;
  if constexpr (DT == 0) {
    float w[4] = {__uint_as_float(raw.x), __uint_as_float(raw.y), __uint_as_float(raw.z), __uint_as_float(raw.w)};
#pragma unroll
    for (int e = 0; e < 4; e++) w[e] = w[e] - lr * g[e] / denom;
    raw = make_uint4(__float_as_uint(w[0]), __float_as_uint(w[1]), __float_as_uint(w[2]), __float_as_uint(w[3]));
  } else {
    uint32_t wd[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      float a = __half2float(__ushort_as_half((unsigned short)(wd[i] & 0xFFFFu)));
      float b = __half2float(__ushort_as_half((unsigned short)(wd[i] >> 16)));
      a = a - lr * g[2 * i] / denom;
      b = b - lr * g[2 * i + 1] / denom;
      wd[i] = (uint32_t)__half_as_ushort(__float2half_rn(a)) | ((uint32_t)__half_as_ushort(__float2half_rn(b)) << 16);
    }
    raw = make_uint4(wd[0], wd[1], wd[2], wd[3]);
  }
  *(uint4 *)wp = raw;
}

struct RowRef {
  char *w;     // the row, where it lives
  float *m;    // its accumulator
};

// The accumulators of all rows stay in HBM (the paper keeps optimizer parameters there,
// Section 5.6.1): only the row itself is in a cache line or in the backing tier.
__device__ inline RowRef locate(const TableMeta &m, uint32_t key, int slot, char *ovf, uint32_t ovf_stride) {
  RowRef r;
  r.w = slot >= 0 ? m.lines + (size_t)(slot - m.slot_base) * m.row_bytes : ovf + (size_t)(-2 - slot) * ovf_stride;
  r.m = m.dev_m + row_of_key(m, key);
  return r;
}

// Sum of the output gradients of the lookups [i0, i1) of one row, as seen by one group of G
// lanes: the bag ids are read G at a time (coalesced) and handed round by shuffles, four
// gradient rows are in flight per lane.  `stride_chunks` > 1 lets several groups share a
// range chunk-wise (group `first_chunk` of `stride_chunks`).  Summation order is fixed.
template <int DT, int G>
__device__ inline void reduce_grads(float (&g)[Elems<DT>::n], const float *gbase, const int32_t *sorted_bag, int bag0,
                                    int sum_dim, int i0, int i1, int first_chunk, int stride_chunks, int lig,
                                    bool active) {
  constexpr int EPL = Elems<DT>::n;
  for (int base = i0 + first_chunk * G; base < i1; base += stride_chunks * G) {
    const int nq = (i1 - base) < G ? (i1 - base) : G;
    const int my_bag = lig < nq ? sorted_bag[base + lig] - bag0 : 0;
    for (int q = 0; q < nq; q += 4) {
      float4 v[4][EPL / 4];
#pragma unroll
      for (int x = 0; x < 4; x++) {
        const int bq = __shfl(my_bag, (q + x) & (G - 1), G);
        const float *p = gbase + (size_t)bq * sum_dim;
        const bool ok = active && (q + x < nq);
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) v[x][e] = ok ? *(const float4 *)(p + 4 * e) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int x = 0; x < 4; x++)
#pragma unroll
        for (int e = 0; e < EPL / 4; e++) {
          g[4 * e] += v[x][e].x; g[4 * e + 1] += v[x][e].y; g[4 * e + 2] += v[x][e].z; g[4 * e + 3] += v[x][e].w;
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

// Rows with at most kLongRun lookups: one group of G lanes per distinct row, gradients
// summed in sorted (= ascending bag) order.
template <int DT, int G>
__global__ __launch_bounds__(256) void backward_short_kernel(const TableMeta *__restrict__ tm, int T, int cls, int B,
                                                             int sum_dim, const uint32_t *__restrict__ uniq_key,
                                                             const int32_t *__restrict__ uniq_tab,
                                                             const int32_t *__restrict__ run_off,
                                                             const int32_t *__restrict__ loc_u,
                                                             const int32_t *__restrict__ sorted_bag,
                                                             const float *__restrict__ grad_out,
                                                             float lr, float eps,
                                                             char *__restrict__ ovf, uint32_t ovf_stride,
                                                             const int32_t *__restrict__ table_class,
                                                             const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  if (cnt->err) return;
  const int n_uniq = cnt->n_uniq;
  const int lig = threadIdx.x % G;
  const int n_groups = gridDim.x * (256 / G);
  for (int u = blockIdx.x * (256 / G) + threadIdx.x / G; u < n_uniq; u += n_groups) {
    const int i0 = run_off[u], i1 = run_off[u + 1];
    if (i1 - i0 > kLongRun) continue;
    const uint32_t key = uniq_key[u];
    const int t = uniq_tab[u];
    if (table_class[t] != cls) continue;
    const TableMeta &m = tm[t];
    const bool active = lig * EPL < m.dim;
    float g[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] = 0.f;
    reduce_grads<DT, G>(g, grad_out + m.col + lig * EPL, sorted_bag, t * B, sum_dim, i0, i1, 0, 1, lig, active);
    update_row<DT, G>(m, key, loc_u[u], ovf, ovf_stride, g, lr, eps, lig, active);
  }
}

// Rows with more lookups are cut into segments of kSegment lookups; one block per segment,
// its 256/G groups take chunks of G lookups round robin and their partial sums are added in
// group order through LDS.  A row of one segment is updated at once; otherwise the segment
// sum goes to the row's slots in `partials` and backward_combine_kernel finishes the row.
template <int DT, int G>
__global__ __launch_bounds__(256) void backward_long_kernel(const TableMeta *__restrict__ tm, int T, int cls, int B,
                                                            int sum_dim, const uint32_t *__restrict__ uniq_key,
                                                             const int32_t *__restrict__ uniq_tab,
                                                            const int32_t *__restrict__ run_off,
                                                            const int32_t *__restrict__ loc_u,
                                                            const int32_t *__restrict__ sorted_bag,
                                                            const uint4 *__restrict__ items,
                                                            const float *__restrict__ grad_out,
                                                            float *__restrict__ partials,
                                                            int pstride, float lr, float eps,
                                                            char *__restrict__ ovf, uint32_t ovf_stride,
                                                             const int32_t *__restrict__ table_class,
                                                            const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  constexpr int NG = 256 / G;
  __shared__ float part[NG][G * EPL + 1];
  if (cnt->err) return;
  const int n_items = cnt->n_items;
  const int lig = threadIdx.x % G, grp = threadIdx.x / G;
  for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
    const uint4 item = items[it];  // (distinct row, segment, segments of the row, first partial slot)
    const int u = (int)item.x;
    const uint32_t key = uniq_key[u];
    const int t = uniq_tab[u];
    if (table_class[t] != cls) continue;  // uniform over the block
    const TableMeta &m = tm[t];
    const bool active = lig * EPL < m.dim;
    const int i0 = run_off[u] + (int)item.y * kSegment;
    const int i1 = min(run_off[u + 1], i0 + kSegment);
    float g[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] = 0.f;
    reduce_grads<DT, G>(g, grad_out + m.col + lig * EPL, sorted_bag, t * B, sum_dim, i0, i1, grp, NG, lig, active);
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
      if (item.z == 1u) {
        update_row<DT, G>(m, key, loc_u[u], ovf, ovf_stride, g, lr, eps, lig, active);
      } else if (active) {
        float *p = partials + (size_t)(item.w + item.y) * pstride + lig * EPL;
#pragma unroll
        for (int e = 0; e < EPL; e++) p[e] = g[e];
      }
    }
  }
}

// Rows of several segments: add the segment sums in segment order, then update the row.
template <int DT, int G>
__global__ __launch_bounds__(256) void backward_combine_kernel(const TableMeta *__restrict__ tm, int T, int cls,
                                                               const uint32_t *__restrict__ uniq_key,
                                                             const int32_t *__restrict__ uniq_tab,
                                                               const int32_t *__restrict__ loc_u,
                                                               const uint4 *__restrict__ huge,
                                                               const float *__restrict__ partials, int pstride,
                                                               float lr, float eps,
                                                               char *__restrict__ ovf, uint32_t ovf_stride,
                                                             const int32_t *__restrict__ table_class,
                                                               const BatchCounters *cnt) {
  constexpr int EPL = Elems<DT>::n;
  if (cnt->err) return;
  const int n_huge = cnt->n_huge;
  const int lig = threadIdx.x % G;
  const int n_groups = gridDim.x * (256 / G);
  for (int hi = blockIdx.x * (256 / G) + threadIdx.x / G; hi < n_huge; hi += n_groups) {
    const uint4 row = huge[hi];  // (distinct row, first partial slot, segments, -)
    const int u = (int)row.x;
    const uint32_t key = uniq_key[u];
    const int t = uniq_tab[u];
    if (table_class[t] != cls) continue;
    const TableMeta &m = tm[t];
    const bool active = lig * EPL < m.dim;
    float g[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) g[e] = 0.f;
    if (active)
      for (uint32_t sgm = 0; sgm < row.z; sgm++) {
        const float *p = partials + (size_t)(row.y + sgm) * pstride + lig * EPL;
#pragma unroll
        for (int e = 0; e < EPL; e++) g[e] += p[e];
      }
    update_row<DT, G>(m, key, loc_u[u], ovf, ovf_stride, g, lr, eps, lig, active);
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
  hipLaunchKernelGGL((forward_kernel<DT, G>), grid, dim3(256), 0, s, tm, tables, b.batch, g.sum_dim, b.d_offsets,
                     b.loc, b.ovf, g.ovf_stride, out, b.cnt);
}

template <int DT, int G>
static void bwd_one(int which, const TableMeta *tm, int cls, const int32_t *table_class, const Geometry &g,
                    const BatchBuf &b, const float *grad_out, float *partials, float lr, float eps, hipStream_t s) {
  if (which == 0) {
    hipLaunchKernelGGL((backward_long_kernel<DT, G>), dim3(4096), dim3(256), 0, s, tm, g.T, cls, b.batch, g.sum_dim,
                       b.uniq_key, b.uniq_tab, b.run_off, b.loc_u, b.sorted_bag, b.items, grad_out, partials,
                       g.partial_stride, lr, eps, b.ovf, g.ovf_stride, table_class, b.cnt);
    hipLaunchKernelGGL((backward_combine_kernel<DT, G>), dim3(256), dim3(256), 0, s, tm, g.T, cls, b.uniq_key, b.uniq_tab,
                       b.loc_u,
                       b.huge, partials, g.partial_stride, lr, eps, b.ovf, g.ovf_stride, table_class, b.cnt);
  } else {
    hipLaunchKernelGGL((backward_short_kernel<DT, G>), dim3(4096), dim3(256), 0, s, tm, g.T, cls, b.batch, g.sum_dim,
                       b.uniq_key, b.uniq_tab, b.run_off, b.loc_u, b.sorted_bag, grad_out, lr, eps, b.ovf, g.ovf_stride, table_class, b.cnt);
  }
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

// long_rows selects the segment kernels (rows with more than kLongRun lookups) or the
// group-per-row kernel (all other rows); a step runs both, they touch disjoint rows.
hipError_t launch_backward_classes(bool long_rows, const TableMeta *tm, const ClassInfo &ci, const Geometry &g,
                                   const BatchBuf &b, const float *grad_out, float *partials, float lr, float eps,
                                   hipStream_t s) {
  if (b.n == 0) return hipSuccess;
  for (int c = 0; c < ci.n_classes; c++)
    TBE_DISPATCH(ci.cls_dtype[c], ci.cls_lanes[c],
                 (bwd_one<d, l>(long_rows ? 0 : 1, tm, c, ci.table_class, g, b, grad_out, partials, lr, eps, s)));
  return hipGetLastError();
}

}  // namespace tbe
