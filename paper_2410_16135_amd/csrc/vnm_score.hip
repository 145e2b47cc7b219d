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

// Column sums: a workgroup owns 64 columns and walks all rows.  Thread (c, q) owns 8 adjacent columns
// (one 16-byte load per row: with 8 such threads a row of the strip is one 128-byte line) and the rows
// q, q + 32, ...; the 32 partial sums of a column meet in LDS and one thread stores their total, so
// every sum is written once, by one thread, without atomics.  `vec` = rows are 16-byte aligned;
// otherwise 2-byte loads.
__global__ void __launch_bounds__(256)
abs_colsum_kernel(const unsigned short* __restrict__ W, int64_t out, int64_t in, int64_t ldw, int vec,
                  unsigned long long* __restrict__ colsum) {
  __shared__ unsigned long long part[32][8][8];
  const int c = threadIdx.x & 7, q = threadIdx.x >> 3;
  const int64_t col = ((int64_t)blockIdx.x * 8 + c) * 8;
  const int nc = col >= in ? 0 : (int)((in - col) < 8 ? (in - col) : 8);
  unsigned long long acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (nc > 0) {
    if (vec && nc == 8) {
      constexpr int kU = 4;                                   // rows in flight per thread
      for (int64_t row = q; row < out; row += 32 * kU) {
        uint4 v[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          const int64_t rr = row + 32 * u;
          v[u] = rr < out ? *(const uint4*)(W + rr * ldw + col) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kU; ++u) {
          const unsigned d[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] += sc_fp16_units((unsigned short)(d[e] & 0xFFFFu));
            acc[2 * e + 1] += sc_fp16_units((unsigned short)(d[e] >> 16));
          }
        }
      }
    } else {
      for (int64_t row = q; row < out; row += 32) {
        const unsigned short* p = W + row * ldw + col;
        for (int e = 0; e < nc; ++e) acc[e] += sc_fp16_units(p[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[q][c][e] = acc[e];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int cc = threadIdx.x >> 3, e = threadIdx.x & 7;
    const int64_t gc = (int64_t)blockIdx.x * 64 + threadIdx.x;
    unsigned long long t = 0;
#pragma unroll
    for (int k = 0; k < 32; ++k) t += part[k][cc][e];
    if (gc < in) colsum[gc] = t;
  }
}

// Row sums: one wave per row, lanes stride over the row 8 columns at a time, one reduction at the end.
__global__ void __launch_bounds__(256)
abs_rowsum_kernel(const unsigned short* __restrict__ W, int64_t out, int64_t in, int64_t ldw, int vec,
                  unsigned long long* __restrict__ rowsum) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= out) return;                                    // uniform over the wave
  const unsigned short* p = W + row * ldw;
  unsigned long long acc = 0;
  for (int64_t c = (int64_t)lane * 8; c < in; c += 512) {
    if (vec && c + 8 <= in) {
      const uint4 v = *(const uint4*)(p + c);
      const unsigned d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        acc += sc_fp16_units((unsigned short)(d[e] & 0xFFFFu)) + sc_fp16_units((unsigned short)(d[e] >> 16));
    } else {
      for (int64_t e = c; e < in && e < c + 8; ++e) acc += sc_fp16_units(p[e]);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned lo = __shfl_xor((unsigned)acc, o), hi = __shfl_xor((unsigned)(acc >> 32), o);
    acc += ((unsigned long long)hi << 32) | lo;
  }
  if (lane == 0) rowsum[row] = acc;
}

// Scores: thread t owns 4 adjacent columns (`vec`: one 8-byte load of W and one 16-byte store of S per
// row) and walks the rows blockIdx.y, blockIdx.y + gridDim.y, ...
__global__ void __launch_bounds__(256)
ria_score_kernel(const unsigned short* __restrict__ W, int64_t out, int64_t in, int64_t ldw,
                 const unsigned long long* __restrict__ colsum, const unsigned long long* __restrict__ rowsum,
                 const float* __restrict__ act, float* __restrict__ S, int64_t lds, int vec) {
  const int64_t col = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (col >= in) return;
  const int nc = (int)((in - col) < 4 ? (in - col) : 4);
  unsigned long long cs[4] = {0, 0, 0, 0};
  double cd[4] = {0, 0, 0, 0}, ad[4] = {0, 0, 0, 0};
  for (int e = 0; e < nc; ++e) { cs[e] = colsum[col + e]; cd[e] = (double)cs[e]; ad[e] = (double)act[col + e]; }
  for (int64_t row = blockIdx.y; row < out; row += gridDim.y) {
    const unsigned long long rs = rowsum[row];
    const double rd = (double)rs;
    unsigned short h[4] = {0, 0, 0, 0};
    if (vec && nc == 4) {
      const uint2 v = *(const uint2*)(W + row * ldw + col);
      h[0] = (unsigned short)(v.x & 0xFFFFu); h[1] = (unsigned short)(v.x >> 16);
      h[2] = (unsigned short)(v.y & 0xFFFFu); h[3] = (unsigned short)(v.y >> 16);
    } else {
      for (int e = 0; e < nc; ++e) h[e] = W[row * ldw + col + e];
    }
    float sc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const double a = (double)sc_fp16_units(h[e]);
      const double q_col = cs[e] ? a / cd[e] : 0.0;
      const double q_row = rs ? a / rd : 0.0;
      const double sum = q_col + q_row;
      sc[e] = (float)(sum * ad[e]);
    }
    if (vec && nc == 4) *(float4*)(S + row * lds + col) = make_float4(sc[0], sc[1], sc[2], sc[3]);
    else for (int e = 0; e < nc; ++e) S[row * lds + col + e] = sc[e];
  }
}

int launch_ria_scores(const void* W, int64_t out, int64_t in, int64_t ldw, const void* act, void* S,
                      int64_t lds, void* workspace, hipStream_t st) {
  if ((in + 63) / 64 > 0x7FFFFFFF || (out + 3) / 4 > 0x7FFFFFFF) return VNM_ERR_UNSUPPORTED;
  unsigned long long* colsum = (unsigned long long*)workspace;
  unsigned long long* rowsum = colsum + in;
  const int vec = (ldw % 8 == 0) && (((uintptr_t)W & 15) == 0);
  hipLaunchKernelGGL(abs_colsum_kernel, dim3((unsigned)((in + 63) / 64)), dim3(256), 0, st, (const unsigned short*)W, out, in,
                     ldw, vec, colsum);
  hipLaunchKernelGGL(abs_rowsum_kernel, dim3((unsigned)((out + 3) / 4)), dim3(256), 0, st, (const unsigned short*)W,
                     out, in, ldw, vec, rowsum);
  const int vec_s = (ldw % 4 == 0) && (((uintptr_t)W & 7) == 0) && (lds % 4 == 0) && (((uintptr_t)S & 15) == 0);
  hipLaunchKernelGGL(ria_score_kernel, dim3((unsigned)((in + 1023) / 1024), (unsigned)(out < 65535 ? out : 65535)), dim3(256), 0, st,
                     (const unsigned short*)W, out, in, ldw, colsum, rowsum, (const float*)act, (float*)S, lds, vec_s);
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

// ---------------------------------------------------------------- LoRA merge (Section 4.3, Eq. 10)
// Wm = fp16(W + scale * B A): what the mask update of the second LoRA stage prunes.  So that the
// refreshed mask is reproducible to the bit the arithmetic is pinned down: fp32, one rounding per
// operation (no fused multiply-add), k ascending:
//     acc = 0;  acc = acc + (B[o,k] * A[k,i]);  m = (scale * acc) + W[o,i];  Wm = fp16(m)
// One thread per 8 consecutive columns of 8 consecutive rows (A, r x in fp32, is fetched once per 8
// rows: fetching it once per row made the kernel L2-bound at a third of the speed); W moves with
// 16-byte accesses, B[o, :] is uniform over the threads of a row.
namespace vnm {

constexpr int kMergeRows = 8;   // rows per thread: A is fetched once per 8 rows instead of once per row

__global__ void __launch_bounds__(256)
lora_merge_kernel(const unsigned short* __restrict__ W, int64_t ldw, const float* __restrict__ B, int64_t ldb,
                  const float* __restrict__ A, int64_t lda, int r, float scale, int64_t out, int64_t in,
                  unsigned short* __restrict__ Wm, int64_t ldm, int vec, int avec) {
  // every product and sum below is rounded on its own: no contraction into fused multiply-adds
#pragma clang fp contract(off)
  const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t o0 = ((int64_t)blockIdx.y + (int64_t)blockIdx.z * 65535) * kMergeRows;
  const int64_t i0 = chunk * 8;
  if (o0 >= out || i0 >= in) return;
  const int n = (int)(in - i0 < 8 ? in - i0 : 8);
  const int rows = (int)(out - o0 < kMergeRows ? out - o0 : kMergeRows);
  float acc[kMergeRows][8];
#pragma unroll
  for (int v = 0; v < kMergeRows; ++v)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[v][e] = 0.f;
  for (int k = 0; k < r; ++k) {
    float a[8];
    if (n == 8 && avec) {
      const float4 a0 = *(const float4*)(A + (int64_t)k * lda + i0), a1 = *(const float4*)(A + (int64_t)k * lda + i0 + 4);
      a[0] = a0.x; a[1] = a0.y; a[2] = a0.z; a[3] = a0.w; a[4] = a1.x; a[5] = a1.y; a[6] = a1.z; a[7] = a1.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = e < n ? A[(int64_t)k * lda + i0 + e] : 0.f;
    }
#pragma unroll
    for (int v = 0; v < kMergeRows; ++v) {
      const float b = B[(v < rows ? o0 + v : o0) * ldb + k];      // rows beyond `out` repeat row o0; never stored
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float p = b * a[e]; acc[v][e] = acc[v][e] + p; }
    }
  }
#pragma unroll
  for (int v = 0; v < kMergeRows; ++v) {
    if (v >= rows) break;
    const int64_t o = o0 + v;
    unsigned short w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (vec && n == 8) *(uint4*)w = *(const uint4*)(W + o * ldw + i0);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) if (e < n) w[e] = W[o * ldw + i0 + e];
    }
    unsigned short m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      _Float16 h;
      __builtin_memcpy(&h, &w[e], 2);
      const float sp = scale * acc[v][e];
      const _Float16 res = (_Float16)(sp + (float)h);
      __builtin_memcpy(&m[e], &res, 2);
    }
    if (vec && n == 8) *(uint4*)(Wm + o * ldm + i0) = *(const uint4*)m;
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) if (e < n) Wm[o * ldm + i0 + e] = m[e];
    }
  }
}

int launch_lora_merge(const void* W, int64_t ldw, const void* B, int64_t ldb, const void* A, int64_t lda, int r,
                      float scale, int64_t out, int64_t in, void* Wm, int64_t ldm, hipStream_t st) {
  const int vec = (ldw % 8 == 0) && (ldm % 8 == 0) && ((((uintptr_t)W | (uintptr_t)Wm) & 15) == 0);
  const int avec = (lda % 4 == 0) && (((uintptr_t)A & 15) == 0);
  const int64_t chunks = (in + 7) / 8;
  const int64_t row_tiles = (out + kMergeRows - 1) / kMergeRows;
  const int64_t gz = (row_tiles + 65534) / 65535;
  if (gz > 65535) return VNM_ERR_UNSUPPORTED;
  dim3 grid((unsigned)((chunks + 255) / 256), (unsigned)(row_tiles < 65535 ? row_tiles : 65535), (unsigned)gz);
  hipLaunchKernelGGL(lora_merge_kernel, grid, dim3(256), 0, st, (const unsigned short*)W, ldw, (const float*)B, ldb,
                     (const float*)A, lda, r, scale, out, in, (unsigned short*)Wm, ldm, vec, avec);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "lora_merge_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
