// Importance scores other than |w| (Section 3, step 1): the RIA criterion of Eq. 1 as an fp32 score
// matrix, and the pruning operator of Section 3 driven by any such matrix.
//
// Reproducibility is part of the contract, because a score decides an integer (which column, which
// weight survives): the two sums of Eq. 1 are exact integers (fp16 magnitudes in units of 2^-24, at
// most 2^40 each, summed in 64 bits), every later step is a single IEEE fp64 operation -- convert,
// divide, divide, add, multiply -- and the result is rounded once to fp32.  In the pruning kernel
// the column L1 norms of the scores are added in fp64 one row after the other, a fixed order.
#include "vnm_internal.h"

namespace vnm {

__device__ __forceinline__ unsigned long long sc_fp16_units(unsigned short h) {
  const unsigned bits = h & 0x7FFFu;
  const unsigned e = bits >> 10, m = bits & 0x3FFu;
  return e ? ((unsigned long long)(1024u + m) << (e - 1)) : (unsigned long long)m;
}

__global__ void __launch_bounds__(256) fill_u64_kernel(unsigned long long* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

// One workgroup: 64 rows x 256 columns of W.  Thread t owns column t of the tile and adds its 64
// magnitudes; the row sums of the tile are reduced per wave.  Both go to global memory with 64-bit
// integer atomics (exact, so the order is immaterial).
__global__ void __launch_bounds__(256)
abs_sums_kernel(const unsigned short* __restrict__ W, int64_t out, int64_t in, int64_t ldw,
                unsigned long long* __restrict__ colsum, unsigned long long* __restrict__ rowsum) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t col = (int64_t)blockIdx.x * 256 + tid;
  const int64_t row0 = (int64_t)blockIdx.y * 64;
  unsigned long long csum = 0;
  for (int v = 0; v < 64; ++v) {
    const int64_t row = row0 + v;
    if (row >= out) break;                                   // uniform over the workgroup
    unsigned long long u = 0;
    if (col < in) u = sc_fp16_units(W[row * ldw + col]);
    csum += u;
    // sum over the 64 lanes of the wave
    unsigned long long r = u;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned lo = __shfl_xor((unsigned)r, o), hi = __shfl_xor((unsigned)(r >> 32), o);
      r += ((unsigned long long)hi << 32) | lo;
    }
    if (lane == 0 && r) atomicAdd(rowsum + row, r);
  }
  if (col < in && csum) atomicAdd(colsum + col, csum);
}

__global__ void __launch_bounds__(256)
ria_score_kernel(const unsigned short* __restrict__ W, int64_t out, int64_t in, int64_t ldw,
                 const unsigned long long* __restrict__ colsum, const unsigned long long* __restrict__ rowsum,
                 const float* __restrict__ act, float* __restrict__ S, int64_t lds) {
  const int64_t col = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (col >= in) return;
  const unsigned long long cs = colsum[col];
  const double cd = (double)cs, ad = (double)act[col];
  for (int64_t row = blockIdx.y; row < out; row += gridDim.y) {
    const unsigned long long rs = rowsum[row];
    const double a = (double)sc_fp16_units(W[row * ldw + col]);
    const double q_col = cs ? a / cd : 0.0;
    const double q_row = rs ? a / (double)rs : 0.0;
    const double sum = q_col + q_row;
    S[row * lds + col] = (float)(sum * ad);
  }
}

int launch_ria_scores(const void* W, int64_t out, int64_t in, int64_t ldw, const void* act, void* S,
                      int64_t lds, void* workspace, hipStream_t st) {
  if ((in + 255) / 256 > 0x7FFFFFFF || (out + 63) / 64 > 65535) return VNM_ERR_UNSUPPORTED;
  unsigned long long* colsum = (unsigned long long*)workspace;
  unsigned long long* rowsum = colsum + in;
  const int64_t n = in + out;
  hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, colsum, n);
  hipLaunchKernelGGL(abs_sums_kernel, dim3((unsigned)((in + 255) / 256), (unsigned)((out + 63) / 64)), dim3(256), 0,
                     st, (const unsigned short*)W, out, in, ldw, colsum, rowsum);
  hipLaunchKernelGGL(ria_score_kernel, dim3((unsigned)((in + 255) / 256), (unsigned)(out < 65535 ? out : 65535)), dim3(256), 0, st,
                     (const unsigned short*)W, out, in, ldw, colsum, rowsum, (const float*)act, (float*)S, lds);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "ria score kernels"); return VNM_ERR_HIP; }
  return VNM_OK;
}

// ---------------------------------------------------------------- pruning from a score matrix
// Same structure as the general ABS kernel (one workgroup: one row block x a span of NB column
// blocks), but nothing is staged: phase 1 walks the V rows of a score column in order (lanes along
// the columns, so the reads coalesce), phase 3 gathers the 4 scores and 4 weights of a (row, block)
// straight from global memory.  Scores must be finite and non-negative; they are compared through
// their bit patterns, which for such floats orders them by value.
__device__ __forceinline__ unsigned sc_top2_of_4(unsigned g0, unsigned g1, unsigned g2, unsigned g3) {
  unsigned g[4] = {g0, g1, g2, g3};
  int a = 0;
#pragma unroll
  for (int k = 1; k < 4; ++k) if (g[k] > g[a]) a = k;
  int b = (a == 0) ? 1 : 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) if (k != a && k != b && g[k] > g[b]) b = k;
  const int p0 = a < b ? a : b, p1 = a < b ? b : a;
  return (unsigned)p0 | ((unsigned)p1 << 2);
}

__global__ void __launch_bounds__(256)
prune_scored_kernel(const unsigned short* __restrict__ W, int64_t ldw, const float* __restrict__ S, int64_t lds,
                    int64_t out, int64_t in, int V, int M, int64_t B, int NB,
                    unsigned short* __restrict__ values, unsigned char* __restrict__ meta,
                    unsigned char* __restrict__ colidx, unsigned char* __restrict__ mask) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int64_t r = blockIdx.y;
  const int64_t b0 = (int64_t)blockIdx.x * NB;
  const int nb = (int)((B - b0) < NB ? (B - b0) : NB);
  const int ncol = nb * M;
  const int64_t c0 = b0 * M;
  double* sums = (double*)smem;                                   // [NB * M]
  unsigned char* keep = (unsigned char*)(sums + (size_t)NB * M);  // [NB][4]
  unsigned char* nibs = keep + NB * 4;                            // [V][NB]
  const int tid = threadIdx.x;
  // column L1 norms, rows in order
  for (int c = tid; c < ncol; c += 256) {
    const int64_t col = c0 + c;
    double acc = 0.0;
    if (col < in)
      for (int v = 0; v < V; ++v) {
        const int64_t row = r * V + v;
        if (row < out) acc += (double)S[row * lds + col];
      }
    sums[c] = acc;
  }
  __syncthreads();
  // per block the 4 columns of largest norm, ties to the lower index, ascending
  for (int b = tid; b < nb; b += 256) {
    const double* L = sums + b * M;
    unsigned kp[4] = {0, 0, 0, 0}; int nk = 0;
    for (int c = 0; c < M; ++c) {
      const double Lc = L[c];
      int rank = 0;
      for (int o = 0; o < c; ++o) rank += L[o] >= Lc;
      for (int o = c + 1; o < M; ++o) rank += L[o] > Lc;
      if (rank < 4 && nk < 4) kp[nk++] = (unsigned)c;
    }
    for (int k = 0; k < 4; ++k) keep[b * 4 + k] = (unsigned char)kp[k];
    *(uchar4*)(colidx + (r * B + b0 + b) * 4) =
        make_uchar4((unsigned char)kp[0], (unsigned char)kp[1], (unsigned char)kp[2], (unsigned char)kp[3]);
  }
  __syncthreads();
  // per (row, block) the 2 largest scores of the 4 kept columns, ties to the lower position
  const int64_t vrow_elems = 2 * B;
  for (int idx = tid; idx < V * nb; idx += 256) {
    const int v = idx / nb, b = idx - v * nb;
    const int64_t row = r * V + v;
    unsigned g[4]; unsigned short w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t col = c0 + (int64_t)b * M + keep[b * 4 + k];
      const bool ok = row < out && col < in;
      g[k] = ok ? (__float_as_uint(S[row * lds + col]) & 0x7FFFFFFFu) : 0u;
      w[k] = ok ? W[row * ldw + col] : (unsigned short)0;
    }
    const unsigned nib = sc_top2_of_4(g[0], g[1], g[2], g[3]);
    const unsigned short k0 = w[nib & 3], k1 = w[nib >> 2];
    *(unsigned*)(values + row * vrow_elems + 2 * (b0 + b)) = (unsigned)k0 | ((unsigned)k1 << 16);
    nibs[v * NB + b] = (unsigned char)nib;
  }
  __syncthreads();
  const int nbytes = (nb + 1) / 2;                                // b0 is even: bytes do not straddle spans
  const int64_t mrow = (B + 1) / 2;
  for (int idx = tid; idx < V * nbytes; idx += 256) {
    const int v = idx / nbytes, j = idx - v * nbytes;
    const unsigned lo = nibs[v * NB + 2 * j];
    const unsigned hi = (2 * j + 1 < nb) ? nibs[v * NB + 2 * j + 1] : 0u;
    meta[(r * V + v) * mrow + b0 / 2 + j] = (unsigned char)(lo | (hi << 4));
  }
  if (mask) {
    for (int idx = tid; idx < V * ncol; idx += 256) {
      const int v = idx / ncol, c = idx - v * ncol;
      const int64_t row = r * V + v, col = c0 + c;
      if (row < out && col < in) {
        const int b = c / M, ci = c - b * M;
        const unsigned nib = nibs[v * NB + b];
        mask[row * in + col] = (unsigned char)((keep[b * 4 + (nib & 3)] == ci) | (keep[b * 4 + (nib >> 2)] == ci));
      }
    }
  }
}

int launch_prune_scored(const void* W, int64_t ldw, const void* S, int64_t lds, const Dims& d, void* values,
                        void* meta, void* colidx, void* mask, hipStream_t st) {
  int NB = (256 / d.M) & ~1;
  if (NB < 2) NB = 2;
  const size_t lds_bytes = (size_t)NB * d.M * 8 + (size_t)NB * 4 + (size_t)d.V * NB;
  if (lds_bytes > 64 * 1024 || d.R > 65535) return VNM_ERR_UNSUPPORTED;
  dim3 grid((unsigned)((d.B + NB - 1) / NB), (unsigned)d.R);
  hipLaunchKernelGGL(prune_scored_kernel, grid, dim3(256), lds_bytes, st, (const unsigned short*)W, ldw,
                     (const float*)S, lds, d.out, d.in, d.V, d.M, d.B, NB, (unsigned short*)values,
                     (unsigned char*)meta, (unsigned char*)colidx, (unsigned char*)mask);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "prune_scored_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
