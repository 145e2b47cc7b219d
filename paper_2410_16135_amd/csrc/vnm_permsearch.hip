// Search for the channel permutations of Section 4.2 (Eqs. 7-9).
//
// Objective (Eq. 7): the importance that V:N:M pruning retains on the permuted score matrix.
// Alternation (Eqs. 8-9): input permutation for fixed output permutation, then the reverse, both
// starting from the identity.  The paper models each half-step "approximately" as a linear sum
// assignment problem without printing the model; the one used here: a half-step visits the
// in-block positions (slots) in turn; for slot q the channel at position q of every full block is
// lifted out, gain[b][k] = retained importance of block k with the channel lifted from block b in
// its free position, and the assignment maximising the total gain (Hungarian method, on the host)
// is applied.  The identity assignment is the current state, so the objective never decreases.
// Scores are quantised once to integers, q = rint(score * scale) clipped to [0, 2^32 - 1]; every
// sum is then a 64-bit integer and exact whatever the order of the parallel reduction.
//
// What the device does is the gain matrices -- O(B^2 out) and O(R^2 in V) work per slot -- from
// two transposed working copies of the quantised scores:
//   colT [in][out]  column c of S (original column id) over the rows in current output order:
//                   static during an input half-step, where only block membership changes
//   rowM [out][in]  row o of S (original row id) over the columns in current input order:
//                   static during an output half-step
// Input half-step, per slot: for (block k, row block r) the remainder (the M-1 columns left in the
// block) is ranked by column sum; a lifted column enters the kept four iff it beats the remainder's
// 4th column (ties to the lower position), and then the kept set is the remainder's top three plus
// the lifted column, whose per-row contribution is a1 + max(a2, x) with a1 >= a2 the two largest
// scores of the row among the top three and x the lifted column's score.  a2 per row, sum of a1,
// the threshold and the retained sum without the lifted column are precomputed per (k, r); the
// gain kernel then needs one max and one add per (b, k, row).
// Output half-step, per slot: the kept columns of (row block k with the lifted row of block r)
// can be any four of the M, so each (r, k, column block) is evaluated directly from the remainder
// rows held in LDS.
#include <algorithm>
#include <vector>
#include "vnm_internal.h"

namespace vnm {
namespace {

constexpr int kMaxM = 32;

struct PsDims {
  int64_t out, in, lds;
  int V, M;
  int64_t R, B;       // all row / column blocks, a ragged last one included
  int64_t Rf, Bf;     // full blocks: the ones whose channels move
  double scale;
};

__device__ __forceinline__ unsigned quantise(float s, double scale) {
  double q = rint((double)s * scale);
  if (!(q >= 0.0)) q = 0.0;
  if (q > 4294967295.0) q = 4294967295.0;
  return (unsigned)q;
}

// colT[c][o'] = q(S[po[o']][c]) through a 32 x 32 LDS tile (both sides contiguous)
__global__ void __launch_bounds__(256)
build_colT_kernel(const float* __restrict__ S, PsDims d, const int* __restrict__ po, unsigned* __restrict__ colT) {
  __shared__ unsigned tile[32][33];
  const int64_t c0 = (int64_t)blockIdx.x * 32, o0 = (int64_t)blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int j = ty; j < 32; j += 8) {
    const int64_t o = o0 + j, c = c0 + tx;
    tile[j][tx] = (o < d.out && c < d.in) ? quantise(S[(int64_t)po[o] * d.lds + c], d.scale) : 0u;
  }
  __syncthreads();
  for (int j = ty; j < 32; j += 8) {
    const int64_t c = c0 + j, o = o0 + tx;
    if (c < d.in && o < d.out) colT[c * d.out + o] = tile[tx][j];
  }
}

// rowM[o][i'] = q(S[o][pi[i']])
__global__ void __launch_bounds__(256)
build_rowM_kernel(const float* __restrict__ S, PsDims d, const int* __restrict__ pi, unsigned* __restrict__ rowM) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= d.out * d.in) return;
  const int64_t o = id / d.in, i = id - o * d.in;
  rowM[id] = quantise(S[o * d.lds + pi[i]], d.scale);
}

// colL1[c][r] = sum of colT[c] over row block r
__global__ void __launch_bounds__(256)
col_l1_kernel(const unsigned* __restrict__ colT, PsDims d, int64_t* __restrict__ colL1) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= d.in * d.R) return;
  const int64_t c = id / d.R, r = id - c * d.R;
  const int64_t o0 = r * d.V, o1 = o0 + d.V < d.out ? o0 + d.V : d.out;
  int64_t s = 0;
  for (int64_t o = o0; o < o1; ++o) s += colT[c * d.out + o];
  colL1[id] = s;
}

// Input half-step, per (block k, row block r): rank the remainder of block k.
__global__ void __launch_bounds__(128)
in_precompute_kernel(const unsigned* __restrict__ colT, const int64_t* __restrict__ colL1, PsDims d,
                     const int* __restrict__ member, int slot, int64_t* __restrict__ thrL,
                     int* __restrict__ thrP, int64_t* __restrict__ base, int64_t* __restrict__ sa1,
                     unsigned* __restrict__ a2) {
  const int64_t id = (int64_t)blockIdx.x * 128 + threadIdx.x;
  if (id >= d.Bf * d.R) return;
  const int64_t k = id / d.R, r = id - k * d.R;
  // the four best remainder columns by (column sum descending, position ascending)
  int bp[4] = {-1, -1, -1, -1};
  int64_t bl[4] = {-1, -1, -1, -1};
  for (int p = 0; p < d.M; ++p) {
    if (p == slot) continue;
    const int64_t L = colL1[(int64_t)member[k * d.M + p] * d.R + r];
    int at = 4;
    while (at > 0 && (bp[at - 1] < 0 || L > bl[at - 1])) --at;    // strict: an earlier position wins a tie
    if (at < 4) {
      for (int q = 3; q > at; --q) { bp[q] = bp[q - 1]; bl[q] = bl[q - 1]; }
      bp[at] = p; bl[at] = L;
    }
  }
  const bool has4 = bp[3] >= 0;
  thrL[id] = has4 ? bl[3] : -1;
  thrP[id] = has4 ? bp[3] : 0;
  const unsigned* c0 = colT + (int64_t)member[k * d.M + bp[0]] * d.out;
  const unsigned* c1 = colT + (int64_t)member[k * d.M + bp[1]] * d.out;
  const unsigned* c2 = colT + (int64_t)member[k * d.M + bp[2]] * d.out;
  const unsigned* c3 = has4 ? colT + (int64_t)member[k * d.M + bp[3]] * d.out : c0;
  const int64_t o0 = r * d.V, o1 = o0 + d.V < d.out ? o0 + d.V : d.out;
  int64_t s1 = 0, sb = 0;
  for (int64_t o = o0; o < o1; ++o) {
    const unsigned x0 = c0[o], x1 = c1[o], x2 = c2[o];
    const unsigned hi01 = x0 > x1 ? x0 : x1, lo01 = x0 > x1 ? x1 : x0;
    const unsigned m1 = hi01 > x2 ? hi01 : x2;                              // largest of three
    const unsigned m2 = hi01 > x2 ? (lo01 > x2 ? lo01 : x2) : hi01;         // second largest
    s1 += m1;
    a2[k * d.out + o] = m2;
    if (has4) {
      const unsigned x3 = c3[o];
      sb += (int64_t)m1 + (m2 > x3 ? m2 : x3);                              // two largest of four
    }
  }
  sa1[id] = s1;
  base[id] = sb;
}

// gain[b][k] over a tile of 16 b x 16 k per workgroup, one thread per pair, row blocks in sequence.
__global__ void __launch_bounds__(256)
in_gain_kernel(const unsigned* __restrict__ colT, const int64_t* __restrict__ colL1, PsDims d,
               const int* __restrict__ member, int slot, const int64_t* __restrict__ thrL,
               const int* __restrict__ thrP, const int64_t* __restrict__ base,
               const int64_t* __restrict__ sa1, const unsigned* __restrict__ a2, int64_t* __restrict__ gain) {
  extern __shared__ unsigned lds_u[];
  const int V = d.V, P = V + 1;
  unsigned* la2 = lds_u;               // [16 k][V + 1]
  unsigned* lx = lds_u + 16 * P;       // [16 b][V + 1]
  const int tid = threadIdx.x, kl = tid >> 4, bl = tid & 15;
  const int64_t k = (int64_t)blockIdx.x * 16 + kl, b = (int64_t)blockIdx.y * 16 + bl;
  const bool valid = k < d.Bf && b < d.Bf;
  const int64_t cand = b < d.Bf ? member[b * d.M + slot] : 0;
  int64_t g = 0;
  for (int64_t r = 0; r < d.R; ++r) {
    const int64_t o0 = r * V;
    const int rows = (int)(o0 + V < d.out ? V : d.out - o0);
    __syncthreads();
    for (int e = tid; e < 16 * V; e += 256) {
      const int j = e / V, v = e - j * V;
      const int64_t kk = (int64_t)blockIdx.x * 16 + j, bb = (int64_t)blockIdx.y * 16 + j;
      la2[j * P + v] = (kk < d.Bf && v < rows) ? a2[kk * d.out + o0 + v] : 0u;
      lx[j * P + v] = (bb < d.Bf && v < rows) ? colT[(int64_t)member[bb * d.M + slot] * d.out + o0 + v] : 0u;
    }
    __syncthreads();
    if (!valid) continue;
    const int64_t Lc = colL1[cand * d.R + r];
    const int64_t tl = thrL[k * d.R + r];
    const bool enters = Lc > tl || (Lc == tl && slot < thrP[k * d.R + r]);
    if (!enters) { g += base[k * d.R + r]; continue; }
    uint64_t s = 0;
    for (int v = 0; v < rows; ++v) {
      const unsigned m2 = la2[kl * P + v], x = lx[bl * P + v];
      s += m2 > x ? m2 : x;
    }
    g += sa1[k * d.R + r] + (int64_t)s;
  }
  if (valid) gain[b * d.Bf + k] = g;
}

// Output half-step: Lrem[k][i] = column sums of row block k without its row at `slot`
__global__ void __launch_bounds__(256)
out_precompute_kernel(const unsigned* __restrict__ rowM, PsDims d, const int* __restrict__ member, int slot,
                      int64_t* __restrict__ Lrem) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x, k = blockIdx.y;
  if (i >= d.in) return;
  int64_t s = 0;
  for (int p = 0; p < d.V; ++p)
    if (p != slot) s += rowM[(int64_t)member[k * d.V + p] * d.in + i];
  Lrem[k * d.in + i] = s;
}

// gain[r][k] += over a chunk of NB column blocks: workgroup (k, chunk); the remainder rows of block
// k over the chunk's columns sit in LDS; items (r, block of the chunk) are spread over the threads.
__global__ void __launch_bounds__(256)
out_gain_kernel(const unsigned* __restrict__ rowM, const int64_t* __restrict__ Lrem, PsDims d,
                const int* __restrict__ member, int slot, int NB, int64_t* __restrict__ gain) {
  extern __shared__ unsigned lds_u[];
  const int V = d.V, M = d.M, W = NB * M, P = W | 1;      // odd row pitch
  unsigned* rem = lds_u;                                   // [V - 1][P]
  unsigned long long* acc = (unsigned long long*)(lds_u + (((size_t)(V - 1) * P + 1) & ~(size_t)1));   // [Rf]
  const int tid = threadIdx.x;
  const int64_t k = blockIdx.x;
  const int64_t col0 = (int64_t)blockIdx.y * W;
  for (int e = tid; e < (V - 1) * W; e += 256) {
    const int pr = e / W, cc = e - pr * W;
    const int p = pr < slot ? pr : pr + 1;                 // remainder row pr is position p of the block
    const int64_t i = col0 + cc;
    rem[pr * P + cc] = i < d.in ? rowM[(int64_t)member[k * V + p] * d.in + i] : 0u;
  }
  for (int64_t r = tid; r < d.Rf; r += 256) acc[r] = 0ull;
  __syncthreads();
  const int64_t nblk = (d.B - (int64_t)blockIdx.y * NB) < NB ? (d.B - (int64_t)blockIdx.y * NB) : NB;
  for (int64_t item = tid; item < d.Rf * nblk; item += 256) {
    const int64_t r = item / nblk;
    const int bl = (int)(item - r * nblk);
    const int64_t crow = (int64_t)member[r * V + slot] * d.in;          // the lifted row of block r
    // the four best columns of the block by (column sum descending, index ascending)
    int bc[4] = {0, 0, 0, 0};
    int64_t bL[4] = {-1, -1, -1, -1};
    unsigned cv[4] = {0, 0, 0, 0};
    for (int c = 0; c < M; ++c) {
      const int64_t i = col0 + bl * M + c;
      const unsigned x = i < d.in ? rowM[crow + i] : 0u;
      const int64_t L = (i < d.in ? Lrem[k * d.in + i] : 0) + x;
      int at = 4;
      while (at > 0 && L > bL[at - 1]) --at;
      if (at < 4) {
        for (int q = 3; q > at; --q) { bc[q] = bc[q - 1]; bL[q] = bL[q - 1]; cv[q] = cv[q - 1]; }
        bc[at] = bl * M + c; bL[at] = L; cv[at] = x;
      }
    }
    auto top2 = [](unsigned x0, unsigned x1, unsigned x2, unsigned x3) -> unsigned long long {
      const unsigned h01 = x0 > x1 ? x0 : x1, l01 = x0 > x1 ? x1 : x0;
      const unsigned h23 = x2 > x3 ? x2 : x3, l23 = x2 > x3 ? x3 : x2;
      const unsigned m1 = h01 > h23 ? h01 : h23;
      const unsigned m2 = h01 > h23 ? (l01 > h23 ? l01 : h23) : (l23 > h01 ? l23 : h01);
      return (unsigned long long)m1 + m2;
    };
    unsigned long long s = top2(cv[0], cv[1], cv[2], cv[3]);
    for (int pr = 0; pr < V - 1; ++pr) {
      const unsigned* row = rem + pr * P;
      s += top2(row[bc[0]], row[bc[1]], row[bc[2]], row[bc[3]]);
    }
    atomicAdd(&acc[r], s);
  }
  __syncthreads();
  for (int64_t r = tid; r < d.Rf; r += 256)
    if (acc[r]) atomicAdd((unsigned long long*)&gain[r * d.Rf + k], acc[r]);
}

// Objective: one thread per (row block, column block) of the permuted matrix, ragged ones included.
__global__ void __launch_bounds__(128)
retained_kernel(const float* __restrict__ S, PsDims d, const int* __restrict__ po, const int* __restrict__ pi,
                unsigned long long* __restrict__ total) {
  const int64_t id = (int64_t)blockIdx.x * 128 + threadIdx.x;
  unsigned long long mine = 0;
  if (id < d.R * d.B) {
    const int64_t r = id / d.B, b = id - r * d.B;
    const int64_t o0 = r * d.V, o1 = o0 + d.V < d.out ? o0 + d.V : d.out;
    int bc[4] = {0, 0, 0, 0};
    int64_t bL[4] = {-1, -1, -1, -1};
    for (int c = 0; c < d.M; ++c) {
      const int64_t i = b * d.M + c;
      int64_t L = 0;
      if (i < d.in) {
        const int64_t src = pi[i];
        for (int64_t o = o0; o < o1; ++o) L += quantise(S[(int64_t)po[o] * d.lds + src], d.scale);
      }
      int at = 4;
      while (at > 0 && L > bL[at - 1]) --at;
      if (at < 4) {
        for (int q = 3; q > at; --q) { bc[q] = bc[q - 1]; bL[q] = bL[q - 1]; }
        bc[at] = c; bL[at] = L;
      }
    }
    for (int64_t o = o0; o < o1; ++o) {
      unsigned m1 = 0, m2 = 0;
      for (int q = 0; q < 4; ++q) {
        const int64_t i = b * d.M + bc[q];
        const unsigned x = i < d.in ? quantise(S[(int64_t)po[o] * d.lds + pi[i]], d.scale) : 0u;
        if (x > m1) { m2 = m1; m1 = x; } else if (x > m2) m2 = x;
      }
      mine += (unsigned long long)m1 + m2;
    }
  }
  // wave reduction, then one atomic per wave
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off, 64);
  if ((threadIdx.x & 63) == 0 && mine) atomicAdd(total, mine);
}

__global__ void fill_i64_kernel(int64_t* p, int64_t n, int64_t v) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// ---- workspace layout (all offsets multiples of 256)
struct PsLayout {
  int64_t po, pi, member, mat, colL1, thrL, thrP, base, sa1, a2, Lrem, gain, total, bytes;
};

PsLayout ps_layout(const PsDims& d) {
  auto up = [](int64_t x) { return (x + 255) / 256 * 256; };
  PsLayout l;
  int64_t off = 0;
  auto take = [&](int64_t bytes) { const int64_t at = off; off += up(bytes); return at; };
  const int64_t n = std::max(d.Bf, d.Rf);
  l.po = take(d.out * 4);
  l.pi = take(d.in * 4);
  l.member = take(std::max(d.Bf * d.M, d.Rf * d.V) * 4);
  l.mat = take(d.out * d.in * 4);                       // colT or rowM
  l.colL1 = take(d.in * d.R * 8);
  l.thrL = take(d.Bf * d.R * 8);
  l.thrP = take(d.Bf * d.R * 4);
  l.base = take(d.Bf * d.R * 8);
  l.sa1 = take(d.Bf * d.R * 8);
  l.a2 = take(d.Bf * d.out * 4);
  l.Lrem = take(d.Rf * d.in * 8);
  l.gain = take(n * n * 8);
  l.total = take(8);
  l.bytes = off;
  return l;
}

int check_hip(hipError_t e, const char* where) {
  if (e == hipSuccess) return VNM_OK;
  set_hip_error(e, where);
  return VNM_ERR_HIP;
}

struct Ctx {
  const float* S;
  PsDims d;
  PsLayout l;
  char* ws;
  hipStream_t st;
  template <typename T> T* at(int64_t off) const { return (T*)(ws + off); }
};

int upload(const Ctx& c, int64_t off, const int* host, int64_t n) {
  if (int rc = check_hip(hipMemcpyAsync(c.ws + off, host, (size_t)n * 4, hipMemcpyHostToDevice, c.st), "hipMemcpyAsync")) return rc;
  return check_hip(hipStreamSynchronize(c.st), "hipStreamSynchronize");   // the host vector may change next
}

int objective(const Ctx& c, int64_t* value) {
  const PsDims& d = c.d;
  hipLaunchKernelGGL(fill_i64_kernel, dim3(1), dim3(256), 0, c.st, c.at<int64_t>(c.l.total), (int64_t)1, (int64_t)0);
  hipLaunchKernelGGL(retained_kernel, dim3((unsigned)((d.R * d.B + 127) / 128)), dim3(128), 0, c.st, c.S, d,
                     c.at<int>(c.l.po), c.at<int>(c.l.pi), c.at<unsigned long long>(c.l.total));
  if (int rc = check_hip(hipGetLastError(), "retained_kernel")) return rc;
  if (int rc = check_hip(hipMemcpyAsync(value, c.ws + c.l.total, 8, hipMemcpyDeviceToHost, c.st), "hipMemcpyAsync")) return rc;
  return check_hip(hipStreamSynchronize(c.st), "hipStreamSynchronize");
}

// state of an input half-step: colT in current output order, column sums per row block
int begin_input_step(const Ctx& c) {
  const PsDims& d = c.d;
  hipLaunchKernelGGL(build_colT_kernel, dim3((unsigned)((d.in + 31) / 32), (unsigned)((d.out + 31) / 32)), dim3(256), 0,
                     c.st, c.S, d, c.at<int>(c.l.po), c.at<unsigned>(c.l.mat));
  hipLaunchKernelGGL(col_l1_kernel, dim3((unsigned)((d.in * d.R + 255) / 256)), dim3(256), 0, c.st,
                     c.at<unsigned>(c.l.mat), d, c.at<int64_t>(c.l.colL1));
  return check_hip(hipGetLastError(), "build_colT_kernel");
}

int gain_input(const Ctx& c, int slot) {
  const PsDims& d = c.d;
  hipLaunchKernelGGL(in_precompute_kernel, dim3((unsigned)((d.Bf * d.R + 127) / 128)), dim3(128), 0, c.st,
                     c.at<unsigned>(c.l.mat), c.at<int64_t>(c.l.colL1), d, c.at<int>(c.l.member), slot,
                     c.at<int64_t>(c.l.thrL), c.at<int>(c.l.thrP), c.at<int64_t>(c.l.base), c.at<int64_t>(c.l.sa1),
                     c.at<unsigned>(c.l.a2));
  const size_t lds = (size_t)2 * 16 * (d.V + 1) * 4;
  hipLaunchKernelGGL(in_gain_kernel, dim3((unsigned)((d.Bf + 15) / 16), (unsigned)((d.Bf + 15) / 16)), dim3(256), lds, c.st,
                     c.at<unsigned>(c.l.mat), c.at<int64_t>(c.l.colL1), d, c.at<int>(c.l.member), slot,
                     c.at<int64_t>(c.l.thrL), c.at<int>(c.l.thrP), c.at<int64_t>(c.l.base), c.at<int64_t>(c.l.sa1),
                     c.at<unsigned>(c.l.a2), c.at<int64_t>(c.l.gain));
  return check_hip(hipGetLastError(), "in_gain_kernel");
}

int begin_output_step(const Ctx& c) {
  const PsDims& d = c.d;
  hipLaunchKernelGGL(build_rowM_kernel, dim3((unsigned)((d.out * d.in + 255) / 256)), dim3(256), 0, c.st, c.S, d,
                     c.at<int>(c.l.pi), c.at<unsigned>(c.l.mat));
  return check_hip(hipGetLastError(), "build_rowM_kernel");
}

int gain_output(const Ctx& c, int slot) {
  const PsDims& d = c.d;
  hipLaunchKernelGGL(out_precompute_kernel, dim3((unsigned)((d.in + 255) / 256), (unsigned)d.Rf), dim3(256), 0, c.st,
                     c.at<unsigned>(c.l.mat), d, c.at<int>(c.l.member), slot, c.at<int64_t>(c.l.Lrem));
  const int64_t n2 = d.Rf * d.Rf;
  hipLaunchKernelGGL(fill_i64_kernel, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, c.st, c.at<int64_t>(c.l.gain), n2,
                     (int64_t)0);
  // column blocks per workgroup: as many as keep the remainder rows below 48 KiB of LDS, at most 16
  int NB = (int)(48 * 1024 / ((int64_t)(d.V - 1) * d.M * 4));
  NB = NB > 16 ? 16 : (NB < 1 ? 1 : NB);
  const size_t rem_words = (((size_t)(d.V - 1) * ((size_t)(NB * d.M) | 1)) + 1) & ~(size_t)1;
  const size_t lds = rem_words * 4 + (size_t)d.Rf * 8;
  if (int rc = allow_big_lds((const void*)out_gain_kernel, "hipFuncSetAttribute(out_gain)")) return rc;
  hipLaunchKernelGGL(out_gain_kernel, dim3((unsigned)d.Rf, (unsigned)((d.B + NB - 1) / NB)), dim3(256), lds, c.st,
                     c.at<unsigned>(c.l.mat), c.at<int64_t>(c.l.Lrem), d, c.at<int>(c.l.member), slot, NB,
                     c.at<int64_t>(c.l.gain));
  return check_hip(hipGetLastError(), "out_gain_kernel");
}

int fetch_gain(const Ctx& c, int64_t n, int64_t* host) {
  if (int rc = check_hip(hipMemcpyAsync(host, c.ws + c.l.gain, (size_t)(n * n) * 8, hipMemcpyDeviceToHost, c.st), "hipMemcpyAsync")) return rc;
  return check_hip(hipStreamSynchronize(c.st), "hipStreamSynchronize");
}

int make_ctx(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M, double scale, void* ws,
             int64_t ws_bytes, void* stream, Ctx* c) {
  if (!S || !ws) return VNM_ERR_NULL;
  if (out <= 0 || in <= 0 || lds < in) return VNM_ERR_SHAPE;
  if (N != 2 || M < 4 || M > kMaxM || !(V == 16 || V == 32 || V == 64 || V == 128)) return VNM_ERR_UNSUPPORTED;
  if (out > 0x7FFFFFFF || in > 0x7FFFFFFF || !(scale > 0.0)) return VNM_ERR_UNSUPPORTED;
  if (((uintptr_t)S & 3) || ((uintptr_t)ws & 255)) return VNM_ERR_ALIGN;
  PsDims d;
  d.out = out; d.in = in; d.lds = lds; d.V = V; d.M = M; d.scale = scale;
  d.R = (out + V - 1) / V; d.B = (in + M - 1) / M; d.Rf = out / V; d.Bf = in / M;
  // grid and LDS limits of the kernels above
  if (d.Rf > 8192 || d.B > 65535 || out / 32 > 65535 || out * in / 256 > 0x7FFFFFFF) return VNM_ERR_UNSUPPORTED;
  c->S = (const float*)S; c->d = d; c->l = ps_layout(d); c->ws = (char*)ws; c->st = (hipStream_t)stream;
  if (ws_bytes < c->l.bytes) return VNM_ERR_WORKSPACE;
  return VNM_OK;
}

bool is_permutation(const int* p, int64_t n) {
  std::vector<char> seen((size_t)n, 0);
  for (int64_t i = 0; i < n; ++i) {
    if (p[i] < 0 || p[i] >= n || seen[(size_t)p[i]]) return false;
    seen[(size_t)p[i]] = 1;
  }
  return true;
}

}  // namespace
}  // namespace vnm

using namespace vnm;

extern "C" int vnm_permutation_search_workspace_bytes(int64_t out, int64_t in, int V, int N, int M, int64_t* bytes) {
  if (!bytes) return VNM_ERR_NULL;
  if (out <= 0 || in <= 0) return VNM_ERR_SHAPE;
  if (N != 2 || M < 4 || M > kMaxM || !(V == 16 || V == 32 || V == 64 || V == 128)) return VNM_ERR_UNSUPPORTED;
  PsDims d;
  d.out = out; d.in = in; d.lds = in; d.V = V; d.M = M; d.scale = 1.0;
  d.R = (out + V - 1) / V; d.B = (in + M - 1) / M; d.Rf = out / V; d.Bf = in / M;
  *bytes = ps_layout(d).bytes;
  return VNM_OK;
}

extern "C" int vnm_retained_score(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M,
                                  double scale, const void* perm_out, const void* perm_in, int64_t* total,
                                  void* workspace, int64_t workspace_bytes, void* stream) {
  if (!total) return VNM_ERR_NULL;
  Ctx c;
  if (int rc = make_ctx(S, out, in, lds, V, N, M, scale, workspace, workspace_bytes, stream, &c)) return rc;
  try {
    std::vector<int> po((size_t)out), pi((size_t)in);
    for (int64_t i = 0; i < out; ++i) po[(size_t)i] = perm_out ? ((const int*)perm_out)[i] : (int)i;
    for (int64_t i = 0; i < in; ++i) pi[(size_t)i] = perm_in ? ((const int*)perm_in)[i] : (int)i;
    if (!is_permutation(po.data(), out) || !is_permutation(pi.data(), in)) return VNM_ERR_SHAPE;
    if (int rc = upload(c, c.l.po, po.data(), out)) return rc;
    if (int rc = upload(c, c.l.pi, pi.data(), in)) return rc;
    return objective(c, total);
  } catch (...) { return VNM_ERR_WORKSPACE; }
}

extern "C" int vnm_permutation_gain(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M,
                                    double scale, int which, int slot, const void* perm_out,
                                    const void* perm_in, void* gain, void* workspace,
                                    int64_t workspace_bytes, void* stream) {
  if (!gain) return VNM_ERR_NULL;
  Ctx c;
  if (int rc = make_ctx(S, out, in, lds, V, N, M, scale, workspace, workspace_bytes, stream, &c)) return rc;
  if ((which != 0 && which != 1) || slot < 0 || slot >= (which == 0 ? M : V)) return VNM_ERR_SHAPE;
  const PsDims& d = c.d;
  if ((which == 0 ? d.Bf : d.Rf) < 1) return VNM_ERR_SHAPE;
  try {
    std::vector<int> po((size_t)out), pi((size_t)in);
    for (int64_t i = 0; i < out; ++i) po[(size_t)i] = perm_out ? ((const int*)perm_out)[i] : (int)i;
    for (int64_t i = 0; i < in; ++i) pi[(size_t)i] = perm_in ? ((const int*)perm_in)[i] : (int)i;
    if (!is_permutation(po.data(), out) || !is_permutation(pi.data(), in)) return VNM_ERR_SHAPE;
    if (int rc = upload(c, c.l.po, po.data(), out)) return rc;
    if (int rc = upload(c, c.l.pi, pi.data(), in)) return rc;
    if (which == 0) {
      if (int rc = upload(c, c.l.member, pi.data(), d.Bf * d.M)) return rc;      // member[b][p] = pi[b M + p]
      if (int rc = begin_input_step(c)) return rc;
      if (int rc = gain_input(c, slot)) return rc;
      return fetch_gain(c, d.Bf, (int64_t*)gain);
    }
    if (int rc = upload(c, c.l.member, po.data(), d.Rf * d.V)) return rc;
    if (int rc = begin_output_step(c)) return rc;
    if (int rc = gain_output(c, slot)) return rc;
    return fetch_gain(c, d.Rf, (int64_t*)gain);
  } catch (...) { return VNM_ERR_WORKSPACE; }
}

extern "C" int vnm_permutation_search(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M,
                                      double scale, int iterations, void* perm_out, void* perm_in,
                                      int64_t* history, void* workspace, int64_t workspace_bytes,
                                      void* stream) {
  if (!perm_out || !perm_in || !history) return VNM_ERR_NULL;
  if (iterations < 0) return VNM_ERR_SHAPE;
  Ctx c;
  if (int rc = make_ctx(S, out, in, lds, V, N, M, scale, workspace, workspace_bytes, stream, &c)) return rc;
  const PsDims& d = c.d;
  int* po = (int*)perm_out;
  int* pi = (int*)perm_in;
  try {
    for (int64_t i = 0; i < out; ++i) po[i] = (int)i;
    for (int64_t i = 0; i < in; ++i) pi[i] = (int)i;
    if (int rc = upload(c, c.l.po, po, out)) return rc;
    if (int rc = upload(c, c.l.pi, pi, in)) return rc;
    if (int rc = objective(c, &history[0])) return rc;
    const int64_t nmax = std::max(d.Bf, d.Rf);
    std::vector<int64_t> gain((size_t)(nmax * nmax));
    std::vector<int> assign((size_t)nmax), lifted((size_t)nmax);
    int h = 1;
    for (int it = 0; it < iterations; ++it) {
      // Eq. 8: input permutation for the current output permutation
      if (d.Bf >= 2) {
        if (int rc = upload(c, c.l.member, pi, d.Bf * d.M)) return rc;
        if (int rc = begin_input_step(c)) return rc;
        for (int slot = 0; slot < M; ++slot) {
          if (int rc = gain_input(c, slot)) return rc;
          if (int rc = fetch_gain(c, d.Bf, gain.data())) return rc;
          int64_t tot = 0;
          if (int rc = vnm_lsa_max(gain.data(), (int)d.Bf, assign.data(), &tot)) return rc;
          for (int64_t b = 0; b < d.Bf; ++b) lifted[(size_t)b] = pi[b * M + slot];
          for (int64_t b = 0; b < d.Bf; ++b) pi[(int64_t)assign[(size_t)b] * M + slot] = lifted[(size_t)b];
          if (int rc = upload(c, c.l.member, pi, d.Bf * d.M)) return rc;
        }
        if (int rc = upload(c, c.l.pi, pi, in)) return rc;
      }
      if (int rc = objective(c, &history[h++])) return rc;
      // Eq. 9: output permutation for the current input permutation
      if (d.Rf >= 2) {
        if (int rc = upload(c, c.l.member, po, d.Rf * d.V)) return rc;
        if (int rc = begin_output_step(c)) return rc;
        for (int slot = 0; slot < V; ++slot) {
          if (int rc = gain_output(c, slot)) return rc;
          if (int rc = fetch_gain(c, d.Rf, gain.data())) return rc;
          int64_t tot = 0;
          if (int rc = vnm_lsa_max(gain.data(), (int)d.Rf, assign.data(), &tot)) return rc;
          for (int64_t r = 0; r < d.Rf; ++r) lifted[(size_t)r] = po[r * V + slot];
          for (int64_t r = 0; r < d.Rf; ++r) po[(int64_t)assign[(size_t)r] * V + slot] = lifted[(size_t)r];
          if (int rc = upload(c, c.l.member, po, d.Rf * d.V)) return rc;
        }
        if (int rc = upload(c, c.l.po, po, out)) return rc;
      }
      if (int rc = objective(c, &history[h++])) return rc;
    }
  } catch (...) { return VNM_ERR_WORKSPACE; }
  return VNM_OK;
}
