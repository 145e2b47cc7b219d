// Linear sum assignment on the host (Section 4.2: each half-step of the permutation search is
// modelled as one and solved with the Hungarian algorithm).
//
// Shortest-augmenting-path form of the Hungarian method with row and column potentials, O(n^3),
// all arithmetic in 64-bit integers (the gains are sums of quantised scores, so the optimum is
// exact).  Maximisation is turned into minimisation of max_gain - gain.
#include <vector>
#include "vnm_internal.h"

extern "C" int vnm_lsa_max(const void* gain_v, int n, void* assign_v, int64_t* total) {
  const int64_t* gain = (const int64_t*)gain_v;
  int* assign = (int*)assign_v;
  if (!gain || !assign || !total) return VNM_ERR_NULL;
  if (n <= 0) return VNM_ERR_SHAPE;
  int64_t gmax = 0;
  for (int64_t i = 0; i < (int64_t)n * n; ++i) {
    if (gain[i] < 0 || gain[i] > (int64_t)1 << 60) return VNM_ERR_SHAPE;
    if (gain[i] > gmax) gmax = gain[i];
  }
  try {
    const int64_t INF = INT64_MAX / 4;
    // 1-based arrays; p[j] = row matched to column j, way[j] = previous column on the path
    std::vector<int64_t> u((size_t)n + 1, 0), v((size_t)n + 1, 0), minv((size_t)n + 1);
    std::vector<int> p((size_t)n + 1, 0), way((size_t)n + 1, 0);
    std::vector<char> used((size_t)n + 1);
    for (int i = 1; i <= n; ++i) {
      p[0] = i;
      int j0 = 0;
      std::fill(minv.begin(), minv.end(), INF);
      std::fill(used.begin(), used.end(), 0);
      do {
        used[(size_t)j0] = 1;
        const int i0 = p[(size_t)j0];
        const int64_t* row = gain + (int64_t)(i0 - 1) * n;
        int64_t delta = INF;
        int j1 = 0;
        for (int j = 1; j <= n; ++j) {
          if (used[(size_t)j]) continue;
          const int64_t cur = (gmax - row[j - 1]) - u[(size_t)i0] - v[(size_t)j];
          if (cur < minv[(size_t)j]) { minv[(size_t)j] = cur; way[(size_t)j] = j0; }
          if (minv[(size_t)j] < delta) { delta = minv[(size_t)j]; j1 = j; }
        }
        for (int j = 0; j <= n; ++j) {
          if (used[(size_t)j]) { u[(size_t)p[(size_t)j]] += delta; v[(size_t)j] -= delta; }
          else minv[(size_t)j] -= delta;
        }
        j0 = j1;
      } while (p[(size_t)j0] != 0);
      do {
        const int j1 = way[(size_t)j0];
        p[(size_t)j0] = p[(size_t)j1];
        j0 = j1;
      } while (j0);
    }
    int64_t sum = 0;
    for (int j = 1; j <= n; ++j) {
      assign[p[(size_t)j] - 1] = j - 1;
      sum += gain[(int64_t)(p[(size_t)j] - 1) * n + (j - 1)];
    }
    *total = sum;
  } catch (...) { return VNM_ERR_WORKSPACE; }                        // out of host memory
  return VNM_OK;
}
