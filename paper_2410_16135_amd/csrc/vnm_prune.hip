// vnm_prune_compress: the pruning operator of Section 3 (ABS score) fused with the conversion to
// the compressed triple of Appendix A.  One workgroup owns one row block and a span of column
// blocks; nothing is exchanged between workgroups.
//
//   phase 0  the V x (NB*M) tile of W is copied to LDS (zero where W is padded)
//   phase 1  one thread per tile column adds the V magnitudes as integers (exact: a finite fp16
//            magnitude is an integer multiple of 2^-24 below 2^40 in those units, so V <= 128 of
//            them fit an int64 with room to spare and the sum has no rounding and no order)
//   phase 2  one thread per block keeps the 4 largest column sums, ties to the lower index
//   phase 3  one thread per (row, block pair) keeps the 2 largest magnitudes among the 4 kept
//            columns (integer compare of the fp16 bit pattern without its sign), ties to the lower
//            position, and writes values / meta; an optional pass writes the dense 0-1 mask
#include "vnm_internal.h"

namespace vnm {

__device__ __forceinline__ unsigned long long fp16_units(unsigned short h) {
  const unsigned bits = h & 0x7FFFu;
  const unsigned e = bits >> 10, m = bits & 0x3FFu;
  return e ? ((unsigned long long)(1024u + m) << (e - 1)) : (unsigned long long)m;
}

// top-2 of 4 magnitudes, (magnitude descending, position ascending); returns p0 | p1 << 2, p0 < p1
__device__ __forceinline__ unsigned top2_of_4(unsigned g0, unsigned g1, unsigned g2, unsigned g3) {
  unsigned g[4] = {g0, g1, g2, g3};
  int a = 0;
#pragma unroll
  for (int k = 1; k < 4; ++k) if (g[k] > g[a]) a = k;
  int b = (a == 0) ? 1 : 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) if (k != a && k != b && g[k] > g[b]) b = k;
  // ties: strict '>' while scanning upwards keeps the lowest position
  const int p0 = a < b ? a : b, p1 = a < b ? b : a;
  return (unsigned)p0 | ((unsigned)p1 << 2);
}

__global__ void __launch_bounds__(256)
prune_compress_kernel(const unsigned short* __restrict__ W, int64_t ldw, int64_t out, int64_t in,
                      int V, int M, int64_t B, int NB,
                      unsigned short* __restrict__ values, unsigned char* __restrict__ meta,
                      unsigned char* __restrict__ colidx, unsigned char* __restrict__ mask) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int r = blockIdx.y;
  const int64_t b0 = (int64_t)blockIdx.x * NB;
  const int nb = (int)((B - b0) < NB ? (B - b0) : NB);          // blocks in this span
  const int ncol = nb * M;                                        // tile columns (padded space)
  const int64_t c0 = b0 * M;
  // LDS carve-up
  unsigned short* tile = (unsigned short*)smem;                   // [V][ncolmax]
  const int pitch = NB * M;
  unsigned long long* sums = (unsigned long long*)(smem + (((size_t)V * pitch * 2 + 15) & ~(size_t)15));
  unsigned char* keep = (unsigned char*)(sums + pitch);           // [NB][4]
  unsigned char* nibs = keep + NB * 4;                            // [V][NB]

  const int tid = threadIdx.x;
  // phase 0
  for (int idx = tid; idx < V * ncol; idx += 256) {
    const int v = idx / ncol, c = idx - v * ncol;
    const int64_t row = (int64_t)r * V + v, col = c0 + c;
    unsigned short h = 0;
    if (row < out && col < in) h = W[row * ldw + col];
    tile[v * pitch + c] = h;
  }
  __syncthreads();
  // phase 1
  for (int c = tid; c < ncol; c += 256) {
    unsigned long long s = 0;
    for (int v = 0; v < V; ++v) s += fp16_units(tile[v * pitch + c]);
    sums[c] = s;
  }
  __syncthreads();
  // phase 2
  for (int b = tid; b < nb; b += 256) {
    const unsigned long long* L = sums + b * M;
    int ch[4] = {-1, -1, -1, -1};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      int best = -1;
      for (int c = 0; c < M; ++c) {
        if (c == ch[0] || c == ch[1] || c == ch[2]) continue;
        if (best < 0 || L[c] > L[best]) best = c;
      }
      ch[k] = best;
    }
    // ascending order (4-element sorting network)
#define VNM_CSWAP(i, j) { if (ch[i] > ch[j]) { int t_ = ch[i]; ch[i] = ch[j]; ch[j] = t_; } }
    VNM_CSWAP(0, 1) VNM_CSWAP(2, 3) VNM_CSWAP(0, 2) VNM_CSWAP(1, 3) VNM_CSWAP(1, 2)
#undef VNM_CSWAP
#pragma unroll
    for (int k = 0; k < 4; ++k) keep[b * 4 + k] = (unsigned char)ch[k];
    *(uchar4*)(colidx + ((int64_t)r * B + b0 + b) * 4) =
        make_uchar4((unsigned char)ch[0], (unsigned char)ch[1], (unsigned char)ch[2], (unsigned char)ch[3]);
  }
  __syncthreads();
  // phase 3: values + nibbles
  const int64_t vrow_elems = 2 * B;
  for (int idx = tid; idx < V * nb; idx += 256) {
    const int v = idx / nb, b = idx - v * nb;
    const unsigned short* trow = tile + v * pitch + b * M;
    const unsigned short w0 = trow[keep[b * 4 + 0]], w1 = trow[keep[b * 4 + 1]],
                         w2 = trow[keep[b * 4 + 2]], w3 = trow[keep[b * 4 + 3]];
    const unsigned nib = top2_of_4(w0 & 0x7FFFu, w1 & 0x7FFFu, w2 & 0x7FFFu, w3 & 0x7FFFu);
    const unsigned short w[4] = {w0, w1, w2, w3};
    const unsigned short k0 = w[nib & 3], k1 = w[nib >> 2];
    const int64_t row = (int64_t)r * V + v;
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
    meta[((int64_t)r * V + v) * mrow + b0 / 2 + j] = (unsigned char)(lo | (hi << 4));
  }
  if (mask) {
    for (int idx = tid; idx < V * ncol; idx += 256) {
      const int v = idx / ncol, c = idx - v * ncol;
      const int64_t row = (int64_t)r * V + v, col = c0 + c;
      if (row < out && col < in) {
        const int b = c / M, ci = c - b * M;
        const unsigned nib = nibs[v * NB + b];
        const unsigned char m = (keep[b * 4 + (nib & 3)] == ci) | (keep[b * 4 + (nib >> 2)] == ci);
        mask[row * in + col] = m;
      }
    }
  }
}

int launch_prune_compress(const void* W, int64_t ldw, const Dims& d, void* values, void* meta,
                          void* colidx, void* mask, hipStream_t st) {
  int NB = (256 / d.M) & ~1;
  if (NB < 2) NB = 2;
  const size_t pitch = (size_t)NB * d.M;
  size_t lds = (((size_t)d.V * pitch * 2 + 15) & ~(size_t)15) + pitch * 8 + (size_t)NB * 4 + (size_t)d.V * NB;
  if (lds > 160 * 1024) return VNM_ERR_UNSUPPORTED;
  if (int rc_lds = allow_big_lds((const void*)prune_compress_kernel, "hipFuncSetAttribute(prune_compress)")) return rc_lds;
  dim3 grid((unsigned)((d.B + NB - 1) / NB), (unsigned)d.R);
  hipLaunchKernelGGL(prune_compress_kernel, grid, dim3(256), lds, st, (const unsigned short*)W, ldw,
                     d.out, d.in, d.V, d.M, d.B, NB, (unsigned short*)values, (unsigned char*)meta,
                     (unsigned char*)colidx, (unsigned char*)mask);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "prune_compress_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
