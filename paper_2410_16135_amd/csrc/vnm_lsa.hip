// Linear sum assignment on the host (Section 4.2: each half-step of the permutation search is
// modelled as one and solved exactly).  Two exact solvers on 64-bit integers:
//
// * Auction with epsilon scaling (the default).  Rows bid for columns: a row without a column takes
//   the one of largest value (gain minus price) and raises its price by its margin over the second
//   best plus eps; the previous owner goes back to the queue.  With the gains multiplied by a power
//   of two above n a complete assignment reached at eps = 1 is optimal (every pair is within eps of
//   its row's best value, so the total is within n of the optimum, less than one unit of gain).  eps starts at 1/64 of the
//   largest gain (column minima taken off first) and shrinks sixfold per phase, prices are kept, and
//   of the assignment those pairs that still satisfy the slackness condition at the smaller eps.
//   Rows are processed one at a time in queue order, so the result does not depend on threads or
//   timing.  On the gain matrices of the search -- dense, all values distinct, a few columns the
//   best place for almost every row -- this needs 60-120 row scans per row where the Hungarian
//   method below needs about 200 per row after its cheap starting phases: 10 times faster at
//   n = 2201.  (Tried on these matrices and not used: candidate lists per row, which values this
//   close to each other invalidate at almost every bid; jumping to eps = 1 early, which costs
//   millions of bids.)  The row scan -- all the solver does -- runs 8 columns per instruction where
//   the CPU has AVX-512.  It gives up, and the Hungarian method takes over, when the scaled values
//   would not fit 61 bits or a bid budget of 2000 n is spent.
// * Hungarian method in its shortest-augmenting-path form with row and column potentials u, v
//   (u[i] + v[j] <= cost(i, j) everywhere, with equality on matched pairs).  Maximisation is turned
//   into minimisation of cost = max_gain - gain.  Augmenting one row costs up to O(n^2), so the rows
//   are first matched as far as two cheap passes get (the starting phases of the Jonker-Volgenant
//   variant of the method): every column is offered to the row that is cheapest for it, then each
//   row left over takes the column that is best for it at current prices, lowering that column's
//   price by its margin over the second best and sending the previous owner back to the queue.  Both
//   keep the invariants above; only the rows still unmatched afterwards go through the exact
//   augmentation, which alone would be correct too.
#include <stdint.h>
#include <vector>
#include "vnm_internal.h"

// the vector row scan exists in the host pass only (this file has no device code, but hipcc parses it
// for the device too)
#if defined(__x86_64__) && !defined(__HIP_DEVICE_COMPILE__)
#define VNM_LSA_X86_HOST 1
#include <immintrin.h>
#else
#define VNM_LSA_X86_HOST 0
#endif

namespace {

// One row scan of the auction: values v[j] = (row[j] << sh) - pp[j]; returns the largest, the second
// largest (equal to the largest if that occurs twice) and the lowest position of the largest.
void scan_top2_scalar(const int64_t* row, const int64_t* pp, int n, int sh, int64_t& v1, int64_t& v2, int& j1) {
  int64_t b1 = INT64_MIN, b2 = INT64_MIN;
  int k1 = -1;
  for (int j = 0; j < n; ++j) {
    const int64_t v = (row[j] << sh) - pp[j];
    if (v > b1) { b2 = b1; b1 = v; k1 = j; }
    else if (v > b2) b2 = v;
  }
  v1 = b1; v2 = b2; j1 = k1;
}

#if VNM_LSA_X86_HOST
// The same with 8 columns per instruction (the scalar loop does about one column per nanosecond and
// the scans are all the solver does).  Pass 1: the maximum.  Pass 2 (the row is in L1 by then): the
// maximum of everything that is not the maximum, how often the maximum occurs, and where first.
__attribute__((target("avx512f")))
void scan_top2_avx512(const int64_t* row, const int64_t* pp, int n, int sh, int64_t& v1, int64_t& v2, int& j1) {
  const __m128i shv = _mm_cvtsi32_si128(sh);
  const __m512i lowest = _mm512_set1_epi64(INT64_MIN);
  __m512i m1 = lowest;
  const int nv = n & ~7;
  for (int j = 0; j < nv; j += 8)
    m1 = _mm512_max_epi64(m1, _mm512_sub_epi64(_mm512_sll_epi64(_mm512_loadu_si512(row + j), shv), _mm512_loadu_si512(pp + j)));
  int64_t b1 = _mm512_reduce_max_epi64(m1);
  for (int j = nv; j < n; ++j) { const int64_t v = (row[j] << sh) - pp[j]; b1 = v > b1 ? v : b1; }
  const __m512i top = _mm512_set1_epi64(b1);
  __m512i m2 = lowest;
  int count = 0, first = n;
  for (int j = 0; j < nv; j += 8) {
    const __m512i v = _mm512_sub_epi64(_mm512_sll_epi64(_mm512_loadu_si512(row + j), shv), _mm512_loadu_si512(pp + j));
    const __mmask8 eq = _mm512_cmpeq_epi64_mask(v, top);
    m2 = _mm512_max_epi64(m2, _mm512_mask_mov_epi64(v, eq, lowest));
    if (eq) {
      count += __builtin_popcount((unsigned)eq);
      if (first == n) first = j + __builtin_ctz((unsigned)eq);
    }
  }
  int64_t b2 = _mm512_reduce_max_epi64(m2);
  for (int j = nv; j < n; ++j) {
    const int64_t v = (row[j] << sh) - pp[j];
    if (v == b1) { ++count; if (first == n) first = j; }
    else if (v > b2) b2 = v;
  }
  v1 = b1; v2 = count >= 2 ? b1 : b2; j1 = first;
}

#endif

typedef void (*ScanFn)(const int64_t*, const int64_t*, int, int, int64_t&, int64_t&, int&);

ScanFn pick_scan() {
#if VNM_LSA_X86_HOST
  __builtin_cpu_init();
  if (__builtin_cpu_supports("avx512f")) return scan_top2_avx512;
#endif
  return scan_top2_scalar;
}

// Auction; false = gave up (nothing written that matters), true = assign and total are set.
// simd = false forces the scalar scan (the two are tested against each other).
bool lsa_auction(const int64_t* gain, int n, int64_t gmax, int* assign, int64_t* total, bool simd) {
  if (n == 1) { assign[0] = 0; *total = gain[0]; return true; }
  // gains are multiplied by a power of two above n: at eps = 1 the total is within n < scale units
  // of the optimum, and totals differ by multiples of scale
  int sh = 1;
  while (((int64_t)1 << sh) <= n) ++sh;
  if (gmax > ((((int64_t)1 << 61) - 1) >> sh)) return false;
  const ScanFn scan = simd ? pick_scan() : scan_top2_scalar;
  // value of column j for row i: (gain[i][j] << sh) - pp[j], pp[j] = (colmin[j] << sh) + price[j]
  std::vector<int64_t> pp((size_t)n);
  int64_t C = 0;
  {
    std::vector<int64_t> cmin(gain, gain + n), cmax(gain, gain + n);
    for (int i = 1; i < n; ++i) {
      const int64_t* row = gain + (int64_t)i * n;
      for (int j = 0; j < n; ++j) {
        if (row[j] < cmin[(size_t)j]) cmin[(size_t)j] = row[j];
        if (row[j] > cmax[(size_t)j]) cmax[(size_t)j] = row[j];
      }
    }
    for (int j = 0; j < n; ++j) {
      pp[(size_t)j] = cmin[(size_t)j] << sh;
      if (cmax[(size_t)j] - cmin[(size_t)j] > C) C = cmax[(size_t)j] - cmin[(size_t)j];
    }
    C <<= sh;
  }
  std::vector<int> owner((size_t)n, -1), col((size_t)n, -1), queue;
  queue.reserve((size_t)n * 4);
  int64_t eps = C / 64;
  if (eps < 1) eps = 1;
  const int64_t budget = (int64_t)2000 * n;
  int64_t bids = 0;
  for (;;) {
    // pairs that are still within eps of their row's best value stay, the rest are released
    queue.clear();
    for (int i = 0; i < n; ++i) {
      if (col[(size_t)i] >= 0) {
        int64_t v1, v2; int j1;
        scan(gain + (int64_t)i * n, pp.data(), n, sh, v1, v2, j1);
        const int j = col[(size_t)i];
        if ((gain[(int64_t)i * n + j] << sh) - pp[(size_t)j] < v1 - eps) { owner[(size_t)j] = -1; col[(size_t)i] = -1; }
      }
      if (col[(size_t)i] < 0) queue.push_back(i);
    }
    for (size_t head = 0; head < queue.size(); ++head) {
      if (++bids > budget) return false;
      const int i = queue[head];
      int64_t v1, v2; int j1;
      scan(gain + (int64_t)i * n, pp.data(), n, sh, v1, v2, j1);
      pp[(size_t)j1] += (v1 - v2) + eps;
      const int prev = owner[(size_t)j1];
      owner[(size_t)j1] = i; col[(size_t)i] = j1;
      if (prev >= 0) { col[(size_t)prev] = -1; queue.push_back(prev); }
    }
    if (eps == 1) break;
    eps /= 6;
    if (eps < 1) eps = 1;
  }
  int64_t sum = 0;
  for (int i = 0; i < n; ++i) { assign[i] = col[(size_t)i]; sum += gain[(int64_t)i * n + col[(size_t)i]]; }
  *total = sum;
  return true;
}

void lsa_hungarian(const int64_t* gain, int n, int64_t gmax, int* assign, int64_t* total) {
  {
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
  }
}

}  // namespace

extern "C" int vnm_lsa_max_method(const void* gain_v, int n, int method, void* assign_v, int64_t* total) {
  const int64_t* gain = (const int64_t*)gain_v;
  int* assign = (int*)assign_v;
  if (!gain || !assign || !total) return VNM_ERR_NULL;
  if (n <= 0) return VNM_ERR_SHAPE;
  if (method != VNM_LSA_AUTO && method != VNM_LSA_HUNGARIAN && method != VNM_LSA_AUCTION && method != VNM_LSA_AUCTION_SCALAR)
    return VNM_ERR_UNSUPPORTED;
  int64_t gmax = 0;
  for (int64_t i = 0; i < (int64_t)n * n; ++i) {
    if (gain[i] < 0 || gain[i] > (int64_t)1 << 60) return VNM_ERR_SHAPE;
    if (gain[i] > gmax) gmax = gain[i];
  }
  try {
    if (method != VNM_LSA_HUNGARIAN && lsa_auction(gain, n, gmax, assign, total, method != VNM_LSA_AUCTION_SCALAR)) return VNM_OK;
    if (method == VNM_LSA_AUCTION || method == VNM_LSA_AUCTION_SCALAR) return VNM_ERR_UNSUPPORTED;
    lsa_hungarian(gain, n, gmax, assign, total);
  } catch (...) { return VNM_ERR_WORKSPACE; }                        // out of host memory
  return VNM_OK;
}

extern "C" int vnm_lsa_max(const void* gain, int n, void* assign, int64_t* total) {
  return vnm_lsa_max_method(gain, n, VNM_LSA_AUTO, assign, total);
}
