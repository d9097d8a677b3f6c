// Embedding table assignment (paper Section 5.6.1, Eq. 6): every table goes to one memory
// type, the tables of a memory type fit its size, the lookup time
//   sum over tables t of traffic_t / bandwidth_{memory(t)}
// is minimal.  The paper hands this to a mixed-integer solver; here it is a depth-first
// branch and bound of its own.  Host code only (nothing here touches the GPU).
//
// Bound: with the tables ordered by traffic per byte and the memory types by bandwidth,
// the best *fractional* assignment of the tables still open pours them, densest first, into
// the fastest memory that has room left (rearrangement inequality: the cost of a byte is
// (traffic per byte) x (1 / bandwidth)).  That is a lower bound for every whole assignment of
// those tables, so a subtree whose bound reaches the incumbent is cut.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/tbe.h"

namespace {

struct Solver {
  int T, M;
  std::vector<int64_t> bytes;    // tables in order of traffic per byte, densest first
  std::vector<double> traffic;
  std::vector<double> inv_bw;    // memory types in order of bandwidth, fastest first
  std::vector<int64_t> rem;      // room left per memory type
  std::vector<int> cur, best;
  double best_t = std::numeric_limits<double>::infinity();
  int64_t nodes = 0, max_nodes = 0;
  bool complete = true;

  // lower bound of the time of tables i.. given the room left
  double bound(int i) const {
    double t = 0.0;
    int m = 0;
    int64_t room = M ? rem[0] : 0;
    for (; i < T; i++) {
      if (bytes[i] == 0) { t += traffic[i] * inv_bw[0]; continue; }
      int64_t b = bytes[i];
      while (b > 0) {
        while (m < M && room == 0) { m++; room = m < M ? rem[m] : 0; }
        if (m == M) return std::numeric_limits<double>::infinity();
        const int64_t x = std::min(b, room);
        t += traffic[i] * ((double)x / (double)bytes[i]) * inv_bw[m];
        b -= x; room -= x;
      }
    }
    return t;
  }

  void greedy() {  // incumbent: densest first into the fastest memory with room
    std::vector<int64_t> r = rem;
    std::vector<int> a(T);
    double t = 0.0;
    for (int i = 0; i < T; i++) {
      int m = 0;
      while (m < M && r[m] < bytes[i]) m++;
      if (m == M) return;
      r[m] -= bytes[i]; a[i] = m; t += traffic[i] * inv_bw[m];
    }
    best = a; best_t = t;
  }

  void dfs(int i, double t) {
    if (i == T) {
      if (t < best_t) { best_t = t; best = cur; }
      return;
    }
    if (++nodes > max_nodes) { complete = false; return; }
    // cut what cannot beat the incumbent by more than rounding noise (this also keeps the
    // search from walking through assignments of equal time)
    if (t + bound(i) >= best_t * (1.0 - 1e-14)) return;
    for (int m = 0; m < M && complete; m++) {
      if (rem[m] < bytes[i]) continue;
      // two memory types with the same bandwidth and the same room left are interchangeable
      if (m > 0 && inv_bw[m] == inv_bw[m - 1] && rem[m] == rem[m - 1]) continue;
      rem[m] -= bytes[i]; cur[i] = m;
      dfs(i + 1, t + traffic[i] * inv_bw[m]);
      rem[m] += bytes[i];
    }
  }
};

}  // namespace

extern "C" int tbe_plan_placement(const tbe_place_table *tables, int32_t num_tables, const tbe_place_memory *mems,
                                  int32_t num_mems, int64_t max_nodes, int32_t *h_memory_of_table, double *h_time,
                                  int32_t *h_optimal) {
  if (!tables || !mems || !h_memory_of_table || num_tables <= 0 || num_mems <= 0) return TBE_EINVAL;
  for (int t = 0; t < num_tables; t++)
    if (tables[t].bytes < 0 || !(tables[t].traffic >= 0.0) || !std::isfinite(tables[t].traffic)) return TBE_EINVAL;
  for (int m = 0; m < num_mems; m++)
    if (mems[m].capacity_bytes < 0 || !(mems[m].bandwidth > 0.0) || !std::isfinite(mems[m].bandwidth)) return TBE_EINVAL;
  const int T = num_tables, M = num_mems;
  std::vector<int> torder(T), morder(M);
  std::iota(torder.begin(), torder.end(), 0);
  std::iota(morder.begin(), morder.end(), 0);
  auto density = [&](int t) {
    return tables[t].bytes == 0 ? std::numeric_limits<double>::infinity() : tables[t].traffic / (double)tables[t].bytes;
  };
  std::stable_sort(torder.begin(), torder.end(), [&](int a, int b) { return density(a) > density(b); });
  std::stable_sort(morder.begin(), morder.end(), [&](int a, int b) { return mems[a].bandwidth > mems[b].bandwidth; });
  Solver s;
  s.T = T; s.M = M;
  s.bytes.resize(T); s.traffic.resize(T); s.inv_bw.resize(M); s.rem.resize(M); s.cur.assign(T, 0);
  for (int i = 0; i < T; i++) { s.bytes[i] = tables[torder[i]].bytes; s.traffic[i] = tables[torder[i]].traffic; }
  for (int m = 0; m < M; m++) { s.inv_bw[m] = 1.0 / mems[morder[m]].bandwidth; s.rem[m] = mems[morder[m]].capacity_bytes; }
  s.max_nodes = max_nodes > 0 ? max_nodes : 5000000;
  s.greedy();
  s.dfs(0, 0.0);
  if (s.best.empty()) {
    return TBE_ELIMIT;  // nothing fits (or nothing was found within max_nodes)
  }
  double t = 0.0;
  for (int i = 0; i < T; i++) h_memory_of_table[torder[i]] = morder[s.best[i]];
  for (int i = 0; i < T; i++) t += tables[i].traffic / mems[h_memory_of_table[i]].bandwidth;  // Eq. 6, table by table
  if (h_time) *h_time = t;
  if (h_optimal) *h_optimal = s.complete ? 1 : 0;
  return TBE_OK;
}
