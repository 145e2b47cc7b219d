// Fast vnm_prune_compress / vnm_decompress for M <= 16 and 16-byte-aligned rows (in % 8 == 0,
// ldw % 8 == 0): one workgroup owns one row block (V rows) and a span of whole K steps (8 column
// blocks each), moves W with 16-byte accesses through an LDS tile, and -- for pruning -- emits the
// canonical triple of Appendix A and the matrix-core copy in the same pass, so W is read once and
// nothing is re-read.  Selection rules and exactness are those of Section 3 as implemented in
// vnm_prune.hip: column L1 norms are exact integer sums of the fp16 magnitudes, ties go to the
// lower index.
#include "vnm_internal.h"

namespace vnm {

// |w| of an fp16 bit pattern as a double.  A column sum of up to 128 such terms spans fewer than 53
// bits, so every partial sum is exact in fp64 and the order of additions does not matter.
__device__ __forceinline__ double fp16_abs_f64(unsigned h) {
  const unsigned short b = (unsigned short)(h & 0x7FFFu);
  _Float16 f;
  __builtin_memcpy(&f, &b, 2);
  return (double)f;
}

// Two largest magnitudes of four, ties to the lower position (Section 3, row-wise N:4 step).
// Each candidate becomes the key (magnitude, 3 - position, sign): distinct keys, larger is better.
// Returns positions p0 < p1 as p0 | p1 << 2 and the two kept fp16 patterns in `pair` (p0 low half).
__device__ __forceinline__ unsigned top2_of_4_f(unsigned w0, unsigned w1, unsigned w2, unsigned w3, unsigned& pair) {
  const unsigned k0 = ((w0 & 0x7FFFu) << 3) | (3u << 1) | (w0 >> 15);
  const unsigned k1 = ((w1 & 0x7FFFu) << 3) | (2u << 1) | (w1 >> 15);
  const unsigned k2 = ((w2 & 0x7FFFu) << 3) | (1u << 1) | (w2 >> 15);
  const unsigned k3 = ((w3 & 0x7FFFu) << 3) | (0u << 1) | (w3 >> 15);
  const unsigned a = max(k0, k1), b = min(k0, k1), c = max(k2, k3), d = min(k2, k3);
  const unsigned m1 = max(a, c);
  const unsigned m2 = max(max(b, d), min(a, c));
  const unsigned pa = 3u - ((m1 >> 1) & 3u), pb = 3u - ((m2 >> 1) & 3u);
  const unsigned va = (m1 >> 3) | ((m1 & 1u) << 15), vb = (m2 >> 3) | ((m2 & 1u) << 15);
  const bool sw = pa > pb;
  const unsigned p0 = sw ? pb : pa, p1 = sw ? pa : pb;
  pair = sw ? (vb | (va << 16)) : (va | (vb << 16));
  return p0 | (p1 << 2);
}

struct PruneFastArgs {
  const unsigned short* W; int64_t ldw, out, in;
  int V, M; int64_t R, B, S;
  int KSW;                 // K steps (8 column blocks each) per workgroup
  int G;                   // row groups that sum columns in parallel
  unsigned short* values; unsigned char* meta; unsigned char* colidx; unsigned char* mask;
  uint4* pa; unsigned short* pidx; unsigned* pcol;   // matrix-core copy or null
};

// LDS layout (dynamic): tile u16 [V][NCP] | part f64 [G][NC] | tot f64 [NC] | keep u32 [NBW] | nibs u8 [V][NBW] (mask only)
__global__ void __launch_bounds__(256) prune_pack_kernel(const PruneFastArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int V = a.V, M = a.M;
  const int64_t r = blockIdx.x;
  const int64_t s_begin = (int64_t)blockIdx.y * a.KSW;
  const int nks = (int)((a.S - s_begin) < a.KSW ? (a.S - s_begin) : a.KSW);
  const int NC = a.KSW * 8 * M, NBW = a.KSW * 8;    // columns / blocks of a full span
  const int64_t c0 = s_begin * 8 * M;
  const int64_t b0 = s_begin * 8;
  const int nbw = (int)((a.B - b0) < nks * 8 ? (a.B - b0) : nks * 8);   // real blocks here
  const int NCP = NC + 8;                           // tile pitch in elements (16-byte rows, skewed banks)
  const int G = a.G;
  unsigned short* tile = (unsigned short*)smem;
  double* part = (double*)(smem + (size_t)V * NCP * 2);
  double* tot = part + (size_t)G * NC;
  unsigned* keep = (unsigned*)(tot + NC);
  unsigned char* nibs = (unsigned char*)(keep + NBW);
  const int tid = threadIdx.x;
  const int chunks = NC / 8;

  // phase 0: W tile -> LDS with 16-byte accesses (zero where W is padded); the same registers feed
  // the partial column sums: thread (g, ch) owns 8 columns and the rows g, g + G, g + 2G, ...
  if (tid < chunks * G) {
    const int g = tid / chunks, ch = tid - g * chunks;
    const int64_t col = c0 + ch * 8;
    const bool col_ok = col < a.in;
    double acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0;
    for (int v = g; v < V; v += 4 * G) {
      uint4 w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int vv = v + u * G;
        const int64_t row = r * V + vv;
        w[u] = make_uint4(0, 0, 0, 0);
        if (vv < V && row < a.out && col_ok) w[u] = *(const uint4*)(a.W + row * a.ldw + col);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int vv = v + u * G;
        if (vv < V) {
          *(uint4*)(tile + (size_t)vv * NCP + ch * 8) = w[u];
          const unsigned d[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] += fp16_abs_f64(d[e] & 0xFFFFu);
            acc[2 * e + 1] += fp16_abs_f64(d[e] >> 16);
          }
        }
      }
    }
    double2* pp = (double2*)(part + (size_t)g * NC + ch * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) pp[e] = make_double2(acc[2 * e], acc[2 * e + 1]);
  }
  __syncthreads();
  // phase 1: column totals
  for (int c = tid; c < NC; c += 256) {
    double t = 0.0;
    for (int g = 0; g < G; ++g) t += part[(size_t)g * NC + c];
    tot[c] = t;
  }
  __syncthreads();
  // phase 2: per block keep the 4 columns of largest L1 norm (ties to the lower index), ascending:
  // column c is kept when fewer than 4 columns beat it
  for (int b = tid; b < NBW; b += 256) {
    double L[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) L[c] = c < M ? tot[b * M + c] : -1.0;
    unsigned kp = 0; int nk = 0;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      int rank = 0;
#pragma unroll
      for (int o = 0; o < 16; ++o) rank += (o < c) ? (L[o] >= L[c]) : (L[o] > L[c]);
      if (c < M && rank < 4) { kp |= (unsigned)c << (8 * nk); ++nk; }
    }
    keep[b] = kp;
    if (b < nbw) *(unsigned*)(a.colidx + (r * a.B + b0 + b) * 4) = kp;
  }
  __syncthreads();
  // phase 3: per (row, block) keep the 2 largest magnitudes of the 4 kept columns, and emit the
  // canonical triple and the matrix-core copy.  An item is one lane of one K step in the layout of
  // the sparse matrix instruction: lane l = i + 32 h holds, for every 32-row tile, row i and the
  // kept pairs of blocks 4h .. 4h+3; 2-bit positions at bits [2e+1 : 2e].
  const int tiles = V / 32 > 0 ? V / 32 : 1;
  const int64_t vrow_elems = 2 * a.B;
  const int64_t mrow = (a.B + 1) / 2;
  const bool v16 = (a.B & 3) == 0;
  for (int item = tid; item < nks * 64; item += 256) {
    const int ks = item >> 6, lane = item & 63;
    const int i = lane & 31, h = lane >> 5;
    const int blk0 = ks * 8 + 4 * h;
    const uint4 kp4 = *(const uint4*)(keep + blk0);
    const unsigned kp[4] = {kp4.x, kp4.y, kp4.z, kp4.w};
    const int64_t rs = r * a.S + s_begin + ks;
    unsigned short ixs[4] = {0, 0, 0, 0};
    for (int at = 0; at < tiles; ++at) {
      const int v = at * 32 + i;
      if (v >= V) break;
      const unsigned short* trow = tile + (size_t)v * NCP + blk0 * M;
      unsigned q[4], ix = 0;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const unsigned short* tb = trow + g * M;
        const unsigned w0 = tb[kp[g] & 255u], w1 = tb[(kp[g] >> 8) & 255u], w2 = tb[(kp[g] >> 16) & 255u],
                       w3 = tb[kp[g] >> 24];
        const unsigned nib = top2_of_4_f(w0, w1, w2, w3, q[g]);
        ix |= nib << (4 * g);
      }
      ixs[at] = (unsigned short)ix;
      const int64_t row = r * V + v;
      unsigned short* vdst = a.values + row * vrow_elems + 2 * (b0 + blk0);
      if (v16 && blk0 + 4 <= nbw) {
        *(uint4*)vdst = make_uint4(q[0], q[1], q[2], q[3]);
      } else {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if (blk0 + g < nbw) *(unsigned*)(vdst + 2 * g) = q[g];
      }
      unsigned char* mdst = a.meta + row * mrow + ((b0 + blk0) >> 1);
      if (blk0 < nbw) mdst[0] = (unsigned char)((ix & 15u) | (blk0 + 1 < nbw ? (ix & 0xF0u) : 0u));
      if (blk0 + 2 < nbw) mdst[1] = (unsigned char)(((ix >> 8) & 15u) | (blk0 + 3 < nbw ? ((ix >> 8) & 0xF0u) : 0u));
      if (a.pa) a.pa[(rs * tiles + at) * 64 + lane] = make_uint4(q[0], q[1], q[2], q[3]);
      if (a.mask) *(unsigned*)(nibs + (size_t)v * NBW + blk0) =
          (ix & 15u) | ((ix & 0xF0u) << 4) | ((ix & 0xF00u) << 8) | ((ix & 0xF000u) << 12);
    }
    if (a.pa && V >= 32) {
      unsigned short* pd = a.pidx + (rs * 64 + lane) * tiles;
      if (tiles == 1) pd[0] = ixs[0];
      else if (tiles == 2) *(unsigned*)pd = (unsigned)ixs[0] | ((unsigned)ixs[1] << 16);
      else *(uint2*)pd = make_uint2((unsigned)ixs[0] | ((unsigned)ixs[1] << 16), (unsigned)ixs[2] | ((unsigned)ixs[3] << 16));
    }
  }
  if (a.pa) {
    for (int idx = tid; idx < nks * 8; idx += 256) {
      const int kq = idx & 3, h = (idx >> 2) & 1, ks = idx >> 3;
      unsigned o = 0;
      for (int m = 0; m < 4; ++m) {
        const int blk = 4 * (m >> 1) + 2 * h + (m & 1);
        const unsigned c = (keep[ks * 8 + blk] >> (8 * kq)) & 255u;
        o |= (unsigned)(blk * M + c) << (8 * m);
      }
      a.pcol[(r * a.S + s_begin + ks) * 8 + h * 4 + kq] = o;
    }
  }
  // phase 4: optional dense 0-1 mask
  if (a.mask) {
    __syncthreads();
    for (int item = tid; item < V * chunks; item += 256) {
      const int v = item / chunks, ch = item - v * chunks;
      const int64_t row = r * V + v, col = c0 + ch * 8;
      if (row < a.out && col < a.in) {
        unsigned char mk[8];
        for (int e = 0; e < 8; ++e) {
          const int c = ch * 8 + e, b = c / M, ci = c - b * M;
          const unsigned nib = nibs[(size_t)v * NBW + b];
          const unsigned kp = keep[b];
          mk[e] = (((kp >> (8 * (nib & 3))) & 255u) == (unsigned)ci) | (((kp >> (8 * (nib >> 2))) & 255u) == (unsigned)ci);
        }
        *(uint2*)(a.mask + row * a.in + col) = *(const uint2*)mk;
      }
    }
  }
}

static int prune_fast_ksw(int V, int M) {
  int k = 8;
  while (k > 1 && (size_t)V * (k * 8 * M + 8) * 2 > 46 * 1024) k >>= 1;
  return k;
}

static size_t prune_fast_lds(int V, int M, int KSW, int G, bool mask) {
  const size_t NC = (size_t)KSW * 8 * M, NBW = (size_t)KSW * 8;
  size_t b = (size_t)V * (NC + 8) * 2;
  b += (size_t)G * NC * 8 + NC * 8 + NBW * 4;
  if (mask) b += (size_t)V * NBW;
  return b;
}

bool prune_fast_applicable(const void* W, int64_t ldw, const Dims& d, const void* mask) {
  return d.M <= 16 && d.V % 32 == 0 && d.V <= 128 && d.in % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)W & 15) == 0 &&
         d.S <= 65535 && (!mask || ((uintptr_t)mask & 7) == 0);
}

int launch_prune_fast(const void* W, int64_t ldw, const Dims& d, void* values, void* meta, void* colidx,
                      void* mask, void* packed, hipStream_t st) {
  PruneFastArgs a;
  a.W = (const unsigned short*)W; a.ldw = ldw; a.out = d.out; a.in = d.in; a.V = d.V; a.M = d.M;
  a.R = d.R; a.B = d.B; a.S = d.S;
  a.KSW = prune_fast_ksw(d.V, d.M);
  const int chunks = a.KSW * d.M;
  a.G = 256 / chunks < d.V ? 256 / chunks : d.V;
  a.values = (unsigned short*)values; a.meta = (unsigned char*)meta; a.colidx = (unsigned char*)colidx;
  a.mask = (unsigned char*)mask;
  a.pa = nullptr; a.pidx = nullptr; a.pcol = nullptr;
  if (packed) {
    const PackedLayout pl = packed_layout(d);
    char* p = (char*)packed;
    a.pa = (uint4*)(p + pl.pa_off); a.pidx = (unsigned short*)(p + pl.pidx_off); a.pcol = (unsigned*)(p + pl.pcol_off);
  }
  const size_t lds = prune_fast_lds(d.V, d.M, a.KSW, a.G, mask != nullptr);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)prune_pack_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute(prune_pack)"); return VNM_ERR_HIP; }
    attr_set = true;
  }
  // row blocks along x: workgroups that share a span of columns' cache lines with their
  // neighbours in y sit R apart in launch order
  dim3 grid((unsigned)d.R, (unsigned)((d.S + a.KSW - 1) / a.KSW));
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
