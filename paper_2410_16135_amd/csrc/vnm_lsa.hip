// Linear sum assignment on the host (Section 4.2: each half-step of the permutation search is
// modelled as one and solved with the Hungarian algorithm).
//
// Hungarian method in its shortest-augmenting-path form with row and column potentials u, v
// (u[i] + v[j] <= cost(i, j) everywhere, with equality on matched pairs), all arithmetic in 64-bit
// integers: the gains are sums of quantised scores, so the optimum is exact.  Maximisation is turned
// into minimisation of cost = max_gain - gain.  Augmenting one row costs up to O(n^2), so the rows
// are first matched as far as two cheap passes get (the starting phases of the Jonker-Volgenant
// variant of the method): every column is offered to the row that is cheapest for it, then each
// row left over takes the column that is best for it at current prices, lowering that column's
// price by its margin over the second best and sending the previous owner back to the queue.  Both
// keep the invariants above; only the rows still unmatched afterwards -- a few per cent on the gain
// matrices of the search -- go through the exact augmentation, which alone would be correct too.
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
    const size_t N = (size_t)n + 1;
    // 1-based: p[j] = row matched to column j (0 = none), q[i] = column matched to row i (0 = none)
    std::vector<int64_t> u(N, 0), v(N, 0), minv(N);
    std::vector<int> p(N, 0), q(N, 0), way(N, 0);
    std::vector<char> used(N);
    auto cost = [&](int i, int j) { return gmax - gain[(int64_t)(i - 1) * n + (j - 1)]; };

    // pass 1: column prices = column minima; a column goes to its cheapest row if that row is free
    {
      std::vector<int> best(N, 1);
      for (int j = 1; j <= n; ++j) v[(size_t)j] = cost(1, j);
      for (int i = 2; i <= n; ++i) {
        const int64_t* row = gain + (int64_t)(i - 1) * n;
        for (int j = 1; j <= n; ++j) {
          const int64_t c = gmax - row[j - 1];
          if (c < v[(size_t)j]) { v[(size_t)j] = c; best[(size_t)j] = i; }
        }
      }
      for (int j = n; j >= 1; --j) {
        const int i = best[(size_t)j];
        if (q[(size_t)i] == 0) { q[(size_t)i] = j; p[(size_t)j] = i; }
      }
    }
    // pass 2: rows left over bid for their best column (two sweeps; displaced owners queue up again)
    if (n >= 2) {
      std::vector<int> todo, next;
      for (int i = 1; i <= n; ++i) if (q[(size_t)i] == 0) todo.push_back(i);
      for (int sweep = 0; sweep < 2 && !todo.empty(); ++sweep) {
        next.clear();
        for (const int i : todo) {
          const int64_t* row = gain + (int64_t)(i - 1) * n;
          int64_t r1 = INF, r2 = INF;
          int j1 = 0, j2 = 0;
          for (int j = 1; j <= n; ++j) {
            const int64_t r = (gmax - row[j - 1]) - v[(size_t)j];
            if (r < r1) { r2 = r1; j2 = j1; r1 = r; j1 = j; }
            else if (r < r2) { r2 = r; j2 = j; }
          }
          int take = j1;
          if (r1 < r2) v[(size_t)j1] -= r2 - r1;                  // the row's margin goes off the price
          else if (p[(size_t)j1] != 0 && p[(size_t)j2] == 0) take = j2;   // equally good and free
          const int owner = p[(size_t)take];
          if (owner != 0) { q[(size_t)owner] = 0; next.push_back(owner); }
          p[(size_t)take] = i; q[(size_t)i] = take;
        }
        todo.swap(next);
      }
    }
    // row potentials that go with these prices; a matched pair that is not tight (cannot happen if
    // the passes above are right) is dissolved rather than trusted
    for (int i = 1; i <= n; ++i) {
      const int64_t* row = gain + (int64_t)(i - 1) * n;
      int64_t m = INF;
      for (int j = 1; j <= n; ++j) {
        const int64_t r = (gmax - row[j - 1]) - v[(size_t)j];
        if (r < m) m = r;
      }
      u[(size_t)i] = m;
      const int j = q[(size_t)i];
      if (j != 0 && cost(i, j) - m - v[(size_t)j] != 0) { p[(size_t)j] = 0; q[(size_t)i] = 0; }
    }
    // exact augmentation of every row still unmatched; way[j] = previous column on the path
    for (int i = 1; i <= n; ++i) {
      if (q[(size_t)i] != 0) continue;
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
        q[(size_t)p[(size_t)j0]] = j0;
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
