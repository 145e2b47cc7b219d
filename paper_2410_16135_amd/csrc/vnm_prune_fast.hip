// Fast vnm_prune_compress / vnm_decompress for M <= 16 and 16-byte-aligned rows (in % 8 == 0,
// ldw % 8 == 0): one workgroup owns one row block (V rows) and a span of whole K steps (8 column
// blocks each), moves W with 16-byte accesses through an LDS tile, and -- for pruning -- emits the
// canonical triple of Appendix A and the matrix-core copy in the same pass, so W is read once and
// nothing is re-read.  Selection rules and exactness are those of Section 3 as implemented in
// vnm_prune.hip: column L1 norms are exact integer sums of the fp16 magnitudes, ties go to the
// lower index.
#include "vnm_internal.h"

namespace vnm {

__device__ __forceinline__ unsigned long long fp16_units_f(unsigned h) {
  const unsigned bits = h & 0x7FFFu;
  const unsigned e = bits >> 10, m = bits & 0x3FFu;
  return e ? ((unsigned long long)(1024u + m) << (e - 1)) : (unsigned long long)m;
}

__device__ __forceinline__ unsigned top2_of_4_f(unsigned g0, unsigned g1, unsigned g2, unsigned g3) {
  // (magnitude descending, position ascending): strict '>' while scanning upwards keeps the lowest
  unsigned a = 0, ga = g0;
  if (g1 > ga) { a = 1; ga = g1; }
  if (g2 > ga) { a = 2; ga = g2; }
  if (g3 > ga) { a = 3; ga = g3; }
  unsigned b = (a == 0) ? 1u : 0u;
  unsigned gb = (a == 0) ? g1 : g0;
  if (a != 1 && b != 1 && g1 > gb) { b = 1; gb = g1; }
  if (a != 2 && b != 2 && g2 > gb) { b = 2; gb = g2; }
  if (a != 3 && b != 3 && g3 > gb) { b = 3; gb = g3; }
  const unsigned p0 = a < b ? a : b, p1 = a < b ? b : a;
  return p0 | (p1 << 2);
}

// LDS layout (dynamic): tile u16 [V][NCP] | sums u64 [G][NC] | keep u8 [NBW][4] | pairs u32 [V][NBW] | nibs u8 [V][NBW]
struct PruneFastArgs {
  const unsigned short* W; int64_t ldw, out, in;
  int V, M; int64_t R, B, S;
  int KSW;                 // K steps per workgroup
  unsigned short* values; unsigned char* meta; unsigned char* colidx; unsigned char* mask;
  uint4* pa; unsigned short* pidx; unsigned* pcol;   // matrix-core copy or null
};

__global__ void __launch_bounds__(256) prune_pack_kernel(const PruneFastArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int V = a.V, M = a.M;
  const int64_t r = blockIdx.y;
  const int64_t s_begin = (int64_t)blockIdx.x * a.KSW;
  const int nks = (int)((a.S - s_begin) < a.KSW ? (a.S - s_begin) : a.KSW);
  const int NCmax = a.KSW * 8 * M, NBWmax = a.KSW * 8;
  const int NC = nks * 8 * M;                       // raw columns of this workgroup (padded space)
  const int64_t c0 = s_begin * 8 * M;
  const int64_t b0 = s_begin * 8;
  const int nbw = (int)((a.B - b0) < nks * 8 ? (a.B - b0) : nks * 8);   // real blocks here
  const int NCP = NCmax + 8;                        // tile pitch in elements (16-byte rows, skewed banks)
  const int G = 256 / NCmax > 0 ? 256 / NCmax : 1;  // row groups for the column sums
  unsigned short* tile = (unsigned short*)smem;
  unsigned long long* sums = (unsigned long long*)(smem + (((size_t)V * NCP * 2 + 15) & ~(size_t)15));
  unsigned char* keep = (unsigned char*)(sums + (size_t)G * NCmax);
  unsigned* pairs = (unsigned*)(keep + (((size_t)NBWmax * 4 + 15) & ~(size_t)15));
  unsigned char* nibs = (unsigned char*)(pairs + (size_t)V * NBWmax);
  const int tid = threadIdx.x;

  // phase 0: W tile -> LDS, 16 bytes per access, zero where W is padded
  const int chunks = NC / 8;
  for (int item = tid; item < V * chunks; item += 256) {
    const int v = item / chunks, ch = item - v * chunks;
    const int64_t row = r * V + v, col = c0 + ch * 8;
    uint4 w = make_uint4(0, 0, 0, 0);
    if (row < a.out && col < a.in) w = *(const uint4*)(a.W + row * a.ldw + col);
    *(uint4*)(tile + (size_t)v * NCP + ch * 8) = w;
  }
  __syncthreads();
  // phase 1: exact column sums, G row groups in parallel
  {
    const int g = tid / NC, c = tid - g * NC;
    if (g < G) {
      const int v0 = (V * g) / G, v1 = (V * (g + 1)) / G;
      unsigned long long acc = 0;
      for (int v = v0; v < v1; ++v) acc += fp16_units_f(tile[(size_t)v * NCP + c]);
      sums[(size_t)g * NCmax + c] = acc;
    }
  }
  __syncthreads();
  // phase 2: per block keep the 4 largest column sums (ties to the lower index), ascending
  for (int b = tid; b < nks * 8; b += 256) {
    unsigned long long L[16];
    for (int c = 0; c < M; ++c) {
      unsigned long long t = 0;
      for (int g = 0; g < G; ++g) t += sums[(size_t)g * NCmax + b * M + c];
      L[c] = t;
    }
    int ch[4] = {-1, -1, -1, -1};
    for (int k = 0; k < 4; ++k) {
      int best = -1;
      for (int c = 0; c < M; ++c) {
        if (c == ch[0] || c == ch[1] || c == ch[2]) continue;
        if (best < 0 || L[c] > L[best]) best = c;
      }
      ch[k] = best;
    }
#define VNM_CSWAP(i, j) { if (ch[i] > ch[j]) { int t_ = ch[i]; ch[i] = ch[j]; ch[j] = t_; } }
    VNM_CSWAP(0, 1) VNM_CSWAP(2, 3) VNM_CSWAP(0, 2) VNM_CSWAP(1, 3) VNM_CSWAP(1, 2)
#undef VNM_CSWAP
    for (int k = 0; k < 4; ++k) keep[b * 4 + k] = (unsigned char)ch[k];
    if (b < nbw)
      *(uchar4*)(a.colidx + (r * a.B + b0 + b) * 4) =
          make_uchar4((unsigned char)ch[0], (unsigned char)ch[1], (unsigned char)ch[2], (unsigned char)ch[3]);
  }
  __syncthreads();
  // phase 3: per (row, block) keep the 2 largest magnitudes of the 4 kept columns
  const int64_t vrow_elems = 2 * a.B;
  for (int idx = tid; idx < V * nks * 8; idx += 256) {
    const int v = idx / (nks * 8), b = idx - v * (nks * 8);
    const unsigned short* trow = tile + (size_t)v * NCP + b * M;
    const unsigned w0 = trow[keep[b * 4 + 0]], w1 = trow[keep[b * 4 + 1]], w2 = trow[keep[b * 4 + 2]],
                   w3 = trow[keep[b * 4 + 3]];
    const unsigned nib = top2_of_4_f(w0 & 0x7FFFu, w1 & 0x7FFFu, w2 & 0x7FFFu, w3 & 0x7FFFu);
    const unsigned p0 = nib & 3, p1 = nib >> 2;
    const unsigned k0 = p0 == 0 ? w0 : p0 == 1 ? w1 : w2;            // p0 <= 2
    const unsigned k1 = p1 == 1 ? w1 : p1 == 2 ? w2 : w3;            // p1 >= 1
    const unsigned pair = k0 | (k1 << 16);
    pairs[(size_t)v * NBWmax + b] = pair;
    nibs[(size_t)v * NBWmax + b] = (unsigned char)nib;
    if (b < nbw) *(unsigned*)(a.values + (r * V + v) * vrow_elems + 2 * (b0 + b)) = pair;
  }
  __syncthreads();
  // phase 4: canonical meta bytes (two blocks per byte; b0 is a multiple of 8)
  {
    const int nbytes = (nbw + 1) / 2;
    const int64_t mrow = (a.B + 1) / 2;
    for (int idx = tid; idx < V * nbytes; idx += 256) {
      const int v = idx / nbytes, j = idx - v * nbytes;
      const unsigned lo = nibs[(size_t)v * NBWmax + 2 * j];
      const unsigned hi = (2 * j + 1 < nbw) ? nibs[(size_t)v * NBWmax + 2 * j + 1] : 0u;
      a.meta[(r * V + v) * mrow + b0 / 2 + j] = (unsigned char)(lo | (hi << 4));
    }
  }
  // phase 5: matrix-core copy.  In a 32-row tile lane l = i + 32 h holds row i; its 8 values are the
  // kept pairs of blocks 4h .. 4h+3 of the K step; 2-bit positions at bits [2e+1 : 2e].
  if (a.pa) {
    const int tiles = V / 32;
    for (int idx = tid; idx < nks * tiles * 64; idx += 256) {
      const int lane = idx & 63;
      const int at = (idx >> 6) % tiles, ks = (idx >> 6) / tiles;
      const int i = lane & 31, h = lane >> 5;
      const int v = at * 32 + i;
      const unsigned* pr = pairs + (size_t)v * NBWmax + ks * 8 + 4 * h;
      const unsigned char* nb = nibs + (size_t)v * NBWmax + ks * 8 + 4 * h;
      uint4 q = make_uint4(pr[0], pr[1], pr[2], pr[3]);
      unsigned ix = (unsigned)nb[0] | ((unsigned)nb[1] << 4) | ((unsigned)nb[2] << 8) | ((unsigned)nb[3] << 12);
      // blocks beyond the last real one: value 0, positions (0, 1)
      for (int g = 0; g < 4; ++g)
        if (ks * 8 + 4 * h + g >= nbw) {
          ((unsigned*)&q)[g] = 0;
          ix = (ix & ~(15u << (4 * g))) | (4u << (4 * g));
        }
      const int64_t rs = r * a.S + s_begin + ks;
      a.pa[(rs * tiles + at) * 64 + lane] = q;
      a.pidx[(rs * 64 + lane) * tiles + at] = (unsigned short)ix;
    }
    for (int idx = tid; idx < nks * 8; idx += 256) {
      const int kq = idx & 3, h = (idx >> 2) & 1, ks = idx >> 3;
      unsigned o = 0;
      for (int m = 0; m < 4; ++m) {
        const int blk = 4 * (m >> 1) + 2 * h + (m & 1);
        const unsigned c = (ks * 8 + blk < nbw) ? keep[(ks * 8 + blk) * 4 + kq] : (unsigned)kq;
        o |= (unsigned)(blk * M + c) << (8 * m);
      }
      a.pcol[(r * a.S + s_begin + ks) * 8 + h * 4 + kq] = o;
    }
  }
  // phase 6: optional dense 0-1 mask
  if (a.mask) {
    for (int item = tid; item < V * chunks; item += 256) {
      const int v = item / chunks, ch = item - v * chunks;
      const int64_t row = r * V + v, col = c0 + ch * 8;
      if (row < a.out && col < a.in) {
        unsigned char mk[8];
        for (int e = 0; e < 8; ++e) {
          const int c = ch * 8 + e, b = c / M, ci = c - b * M;
          const unsigned nib = nibs[(size_t)v * NBWmax + b];
          mk[e] = (keep[b * 4 + (nib & 3)] == ci) | (keep[b * 4 + (nib >> 2)] == ci);
        }
        *(uint2*)(a.mask + row * a.in + col) = *(const uint2*)mk;
      }
    }
  }
}

static size_t prune_fast_lds(int V, int M, int KSW) {
  const size_t NC = (size_t)KSW * 8 * M, NBW = (size_t)KSW * 8;
  const size_t G = 256 / NC > 0 ? 256 / NC : 1;
  size_t b = ((size_t)V * (NC + 8) * 2 + 15) & ~(size_t)15;
  b += G * NC * 8;
  b += (NBW * 4 + 15) & ~(size_t)15;
  b += (size_t)V * NBW * 4 + (size_t)V * NBW;
  return b;
}

bool prune_fast_applicable(const void* W, int64_t ldw, const Dims& d, const void* mask) {
  return d.M <= 16 && d.in % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)W & 15) == 0 && d.R <= 65535 &&
         (!mask || ((uintptr_t)mask & 7) == 0);
}

int launch_prune_fast(const void* W, int64_t ldw, const Dims& d, void* values, void* meta, void* colidx,
                      void* mask, void* packed, hipStream_t st) {
  PruneFastArgs a;
  a.W = (const unsigned short*)W; a.ldw = ldw; a.out = d.out; a.in = d.in; a.V = d.V; a.M = d.M;
  a.R = d.R; a.B = d.B; a.S = d.S;
  a.KSW = 128 / (8 * d.M) > 0 ? 128 / (8 * d.M) : 1;
  a.values = (unsigned short*)values; a.meta = (unsigned char*)meta; a.colidx = (unsigned char*)colidx;
  a.mask = (unsigned char*)mask;
  a.pa = nullptr; a.pidx = nullptr; a.pcol = nullptr;
  if (packed) {
    const PackedLayout pl = packed_layout(d);
    char* p = (char*)packed;
    a.pa = (uint4*)(p + pl.pa_off); a.pidx = (unsigned short*)(p + pl.pidx_off); a.pcol = (unsigned*)(p + pl.pcol_off);
  }
  const size_t lds = prune_fast_lds(d.V, d.M, a.KSW);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)prune_pack_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute(prune_pack)"); return VNM_ERR_HIP; }
    attr_set = true;
  }
  dim3 grid((unsigned)((d.S + a.KSW - 1) / a.KSW), (unsigned)d.R);
  hipLaunchKernelGGL(prune_pack_kernel, grid, dim3(256), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "prune_pack_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

// ---------------------------------------------------------------- decompress
// One workgroup: V rows x a span of column blocks.  The dense tile is assembled in LDS (zero fill,
// then two 2-byte scatters per (row, block)) and written out with 16-byte stores.
__global__ void __launch_bounds__(256)
decompress_fast_kernel(const unsigned short* __restrict__ values, const unsigned char* __restrict__ meta,
                       const unsigned char* __restrict__ colidx, int64_t out, int64_t in, int V, int M,
                       int64_t B, int NBW, unsigned short* __restrict__ Wd, int64_t ldw) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int64_t r = blockIdx.y;
  const int64_t b0 = (int64_t)blockIdx.x * NBW;
  const int nb = (int)((B - b0) < NBW ? (B - b0) : NBW);
  const int NCmax = NBW * M;                      // multiple of 8 (NBW is a multiple of 8)
  const int NCP = NCmax + 8;
  const int64_t c0 = b0 * M;
  unsigned short* tile = (unsigned short*)smem;
  const int tid = threadIdx.x;
  const int chunks = NCmax / 8;
  for (int item = tid; item < V * chunks; item += 256) {
    const int v = item / chunks, ch = item - v * chunks;
    *(uint4*)(tile + (size_t)v * NCP + ch * 8) = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  for (int idx = tid; idx < V * nb; idx += 256) {
    const int v = idx / nb, b = idx - v * nb;
    const int64_t row = r * V + v;
    if (row >= out) continue;
    const uchar4 k4 = *(const uchar4*)(colidx + (r * B + b0 + b) * 4);
    const unsigned char k[4] = {k4.x, k4.y, k4.z, k4.w};
    const unsigned byte = meta[row * ((B + 1) / 2) + ((b0 + b) >> 1)];
    const unsigned nib = ((b0 + b) & 1) ? (byte >> 4) : (byte & 15u);
    const unsigned pair = *(const unsigned*)(values + row * 2 * B + 2 * (b0 + b));
    unsigned short* trow = tile + (size_t)v * NCP + b * M;
    trow[k[nib & 3]] = (unsigned short)(pair & 0xFFFFu);
    trow[k[nib >> 2]] = (unsigned short)(pair >> 16);
  }
  __syncthreads();
  for (int item = tid; item < V * chunks; item += 256) {
    const int v = item / chunks, ch = item - v * chunks;
    const int64_t row = r * V + v, col = c0 + ch * 8;
    if (row < out && col < in) *(uint4*)(Wd + row * ldw + col) = *(const uint4*)(tile + (size_t)v * NCP + ch * 8);
  }
}

bool decompress_fast_applicable(const void* W_out, int64_t ldw, const Dims& d) {
  return d.M <= 16 && d.in % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)W_out & 15) == 0 && d.R <= 65535;
}

int launch_decompress_fast(const void* values, const void* meta, const void* colidx, const Dims& d,
                           void* W_out, int64_t ldw, hipStream_t st) {
  const int NBW = 8 * (128 / (8 * d.M) > 0 ? 128 / (8 * d.M) : 1);
  const size_t lds = (size_t)d.V * (NBW * d.M + 8) * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)decompress_fast_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute(decompress_fast)"); return VNM_ERR_HIP; }
    attr_set = true;
  }
  dim3 grid((unsigned)((d.B + NBW - 1) / NBW), (unsigned)d.R);
  hipLaunchKernelGGL(decompress_fast_kernel, grid, dim3(256), lds, st, (const unsigned short*)values,
                     (const unsigned char*)meta, (const unsigned char*)colidx, d.out, d.in, d.V, d.M, d.B,
                     NBW, (unsigned short*)W_out, ldw);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "decompress_fast_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
