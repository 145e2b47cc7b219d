// Fast vnm_prune_compress / vnm_decompress for M <= 16 and 16-byte-aligned rows (in % 8 == 0,
// ldw % 8 == 0): one workgroup owns one row block (V rows) and a span of whole K steps (8 column
// blocks each), moves W with 16-byte accesses through an LDS tile, and -- for pruning -- emits the
// canonical triple of Appendix A and the matrix-core copy in the same pass, so W is read once and
// nothing is re-read.  Selection rules and exactness are those of Section 3 as implemented in
// vnm_prune.hip: column L1 norms are exact integer sums of the fp16 magnitudes, ties go to the
// lower index.
#include "vnm_internal.h"

namespace vnm {

// |w| of the fp16 bit pattern in the low half of h as a double (the high half is ignored).  The sign
// is dropped on the fp32 value, where it is an operand modifier of the second conversion and costs
// no instruction; the empty asm keeps the compiler from moving it back in front of the first one,
// where it would be a mask.  A column sum of up to 128 such terms spans fewer than 53 bits, so every
// partial sum is exact in fp64 and the order of additions does not matter.
__device__ __forceinline__ double fp16_abs_f64(unsigned h) {
  const unsigned short b = (unsigned short)h;
  _Float16 f;
  __builtin_memcpy(&f, &b, 2);
  float t = (float)f;
  asm("" : "+v"(t));
  return (double)__builtin_fabsf(t);
}

// Two largest magnitudes of four, ties to the lower position (Section 3, row-wise N:4 step).
// w0..w3 are fp16 bit patterns (upper halves zero).  Each candidate becomes the key
// (inverted magnitude | 14 zero bits | position | sign), built with one funnel shift and one XOR:
// the keys are distinct and the two smallest belong to the two largest magnitudes, the lower
// position first among equals.  A second funnel shift turns a key into position << 16 | sign << 15 |
// inverted magnitude, so ordering the two winners by that word orders them by position.
// Returns positions p0 < p1 as p0 | p1 << 2 and the two kept fp16 patterns in `pair` (p0 low half).
__device__ __forceinline__ unsigned top2_of_4_f(unsigned w0, unsigned w1, unsigned w2, unsigned w3, unsigned& pair) {
  const unsigned k0 = __builtin_amdgcn_alignbit(w0, w0, 15) ^ 0xFFFE0000u;
  const unsigned k1 = __builtin_amdgcn_alignbit(w1, w1, 15) ^ 0xFFFE0002u;
  const unsigned k2 = __builtin_amdgcn_alignbit(w2, w2, 15) ^ 0xFFFE0004u;
  const unsigned k3 = __builtin_amdgcn_alignbit(w3, w3, 15) ^ 0xFFFE0006u;
  const unsigned a = min(k0, k1), b = max(k0, k1), c = min(k2, k3), d = max(k2, k3);
  const unsigned m1 = min(a, c);
  const unsigned m2 = min(min(b, d), max(a, c));
  const unsigned e1 = __builtin_amdgcn_alignbit(m1, m1, 17), e2 = __builtin_amdgcn_alignbit(m2, m2, 17);
  const unsigned lo = min(e1, e2), hi = max(e1, e2);
  pair = __builtin_amdgcn_perm(hi, lo, 0x05040100u) ^ 0x7FFF7FFFu;
  return (lo >> 16) | ((hi >> 16) << 2);
}

// The same selection on importance scores handed in (finite, non-negative fp32, compared through
// their bit patterns without the sign): positions p0 < p1 of the two largest, ties to the lower position.
__device__ __forceinline__ unsigned top2_of_4_s(unsigned g0, unsigned g1, unsigned g2, unsigned g3) {
  const unsigned g[4] = {g0, g1, g2, g3};
  int a = 0;
#pragma unroll
  for (int k = 1; k < 4; ++k) if (g[k] > g[a]) a = k;
  int b = (a == 0) ? 1 : 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) if (k != a && k != b && g[k] > g[b]) b = k;
  const int p0 = a < b ? a : b, p1 = a < b ? b : a;
  return (unsigned)p0 | ((unsigned)p1 << 2);
}

struct PruneFastArgs {
  const unsigned short* W; int64_t ldw, out, in;
  int V, M; int64_t R, B, S;
  int KSW;                 // K steps (8 column blocks each) per workgroup
  int G;                   // row groups that sum columns in parallel
  unsigned short* values; unsigned char* meta; unsigned char* colidx; unsigned char* mask;
  uint4* pa; unsigned short* pidx; unsigned* pcol;   // matrix-core copy or null
  const float* Sc; int64_t lds_s;                    // importance scores (SCORED instantiation only)
};

// LDS layout (dynamic): tile u16 [V][NCP = NC + 4] | tot f64 [NC] | keep u32 [NBW] | (SCORED) scores f32 [V][NC + 4]
// SCORED: the selections are driven by the score matrix a.Sc instead of |w| (Section 3, steps 2-3 on
// any importance score, e.g. RIA, Eq. 1): column norms are the fp64 sums of the scores added in row
// order (their value can depend on the order, so it is fixed), step 3 compares the scores; the kept
// values are W's.  The plain instantiation is the kernel of the hot path, unchanged.
template <bool SCORED>
__global__ void __launch_bounds__(256) prune_pack_kernel(const PruneFastArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int V = a.V, M = a.M;
  const int64_t r = blockIdx.y;
  const int64_t s_begin = (int64_t)blockIdx.x * a.KSW;
  const int nks = (int)((a.S - s_begin) < a.KSW ? (a.S - s_begin) : a.KSW);
  const int NC = a.KSW * 8 * M, NBW = a.KSW * 8;    // columns / blocks of a full span
  const int64_t c0 = s_begin * 8 * M;
  const int64_t b0 = s_begin * 8;
  const int nbw = (int)((a.B - b0) < nks * 8 ? (a.B - b0) : nks * 8);   // real blocks here
  // tile pitch in elements: 8-byte rows, and a number of dwords that is 2 mod 4, so that the same
  // column of 32 consecutive rows lies in 32 different banks (phase 2 walks the tile that way)
  const int NCP = NC + 4;
  const int G = a.G;
  unsigned short* tile = (unsigned short*)smem;
  double* tot = (double*)(smem + (size_t)V * NCP * 2);
  unsigned* keep = (unsigned*)(tot + NC);
  float* stile = (float*)(keep + NBW);
  const int NCS = NC + 4;                           // score tile pitch in floats (16-byte rows)
  const int tid = threadIdx.x;
  const int chunks = NC / 8;

  for (int c = tid; c < NC; c += 256) tot[c] = 0.0;
  for (int b = tid; b < NBW; b += 256) keep[b] = 0;
  __syncthreads();
  // phase 0: W tile -> LDS, 16 bytes per load and two 8-byte halves per store (zero where W is padded); the same registers feed
  // the column sums: thread (g, ch) owns 8 columns and the rows g, g + G, g + 2G, ...; the partial
  // sums meet in LDS by atomic adds (exact, so their order is immaterial)
  if (tid < chunks * G) {
    const int g = tid / chunks, ch = tid - g * chunks;
    const int64_t col = c0 + ch * 8;
    const bool col_ok = col < a.in;
    double acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0;
    constexpr int kBatch = 12;
    // rows of this tile that exist in W (none when the 8 columns lie beyond the last one)
    const int64_t rows_left = a.out - r * V;
    const int v_real = !col_ok || rows_left <= 0 ? 0 : (rows_left < V ? (int)rows_left : V);
    // a load address is a base that is the same for the whole workgroup (row r V, column c0) plus a
    // 32-bit offset; the loads carry no predicate: a row beyond the last real one reads the last real
    // one instead and is zeroed afterwards (only workgroups at the lower edge of W have such rows)
    const unsigned ldw2 = (unsigned)a.ldw * 2u;
    const char* tile_src = (const char*)(a.W + r * V * a.ldw + c0);
    for (int vb = 0; vb < V; vb += kBatch * G) {
      const int v = vb + g;
      uint4 w[kBatch];
      if (v_real > 0) {
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int vc = v + u * G < v_real ? v + u * G : v_real - 1;
          w[u] = *(const uint4*)(tile_src + (__umul24((unsigned)vc, ldw2) + (unsigned)ch * 16u));
        }
      }
      if (v_real < V) {
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
          if (v + u * G >= v_real) w[u] = make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int vv = v + u * G;
        if (vv < V) {
          uint2* td = (uint2*)(tile + (size_t)vv * NCP + ch * 8);
          td[0] = make_uint2(w[u].x, w[u].y);
          td[1] = make_uint2(w[u].z, w[u].w);
          const unsigned d[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
          if constexpr (!SCORED) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              acc[2 * e] += fp16_abs_f64(d[e]);
              acc[2 * e + 1] += fp16_abs_f64(d[e] >> 16);
            }
          }
        }
      }
    }
    if constexpr (!SCORED) {
#pragma unroll
      for (int e = 0; e < 8; ++e) unsafeAtomicAdd(tot + ch * 8 + e, acc[e]);
    }
  }
  if constexpr (SCORED) {
    // score tile -> LDS with 16-byte accesses (zero where the matrix is padded), then one thread per
    // column adds its V scores in row order
    const int chunks4 = NC / 4;
    const int G4 = 256 / chunks4;
    if (tid < chunks4 * G4) {
      const int g = tid / chunks4, ch = tid - g * chunks4;
      const int64_t col = c0 + ch * 4;
      for (int v = g; v < V; v += G4) {
        const int64_t row = r * V + v;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < a.out && col < a.in) s = *(const float4*)(a.Sc + row * a.lds_s + col);
        *(float4*)(stile + (size_t)v * NCS + ch * 4) = s;
      }
    }
    __syncthreads();
    for (int c = tid; c < NC; c += 256) {
      double acc = 0.0;
      for (int v = 0; v < V; ++v) acc += (double)stile[(size_t)v * NCS + c];
      tot[c] = acc;
    }
  }
  __syncthreads();
  // phase 1: per block keep the 4 columns of largest L1 norm (ties to the lower index), ascending:
  // column c is kept when fewer than 4 columns beat it.  One thread per (block, column) finds that
  // out and sets bit c of the block's word in `keep` (zero since the start of the kernel); one thread
  // per block then lists the 4 set bits, lowest first, a byte each, in the same word
  {
    const unsigned m_inv = (65536u + M - 1) / M;
    for (int p = tid; p < NBW * M; p += 256) {
      const int b = (int)(((unsigned)p * m_inv) >> 16), c = p - b * M;   // p < 2^12, M <= 16: exact
      const double* L = tot + b * M;
      const double Lc = L[c];
      int rank = 0;
      for (int o = 0; o < M; ++o) {
        const double Lo = L[o];
        rank += o < c ? Lo >= Lc : Lo > Lc;      // o == c: Lc > Lc is false
      }
      if (rank < 4) atomicOr(keep + b, 1u << c);
    }
  }
  __syncthreads();
  for (int b = tid; b < NBW; b += 256) {
    unsigned m = keep[b], kp = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      kp |= (m ? (unsigned)__builtin_ctz(m) : 0u) << (8 * k);   // (fewer than 4 bits only if a norm is not a number)
      m &= m - 1;
    }
    keep[b] = kp;
    if (b < nbw) *(unsigned*)(a.colidx + (r * a.B + b0 + b) * 4) = kp;
  }
  __syncthreads();
  // phase 2: per (row, block) keep the 2 largest magnitudes of the 4 kept columns.  An item is one
  // lane of one K step in the layout of the sparse matrix instruction: lane l = i + 32 h holds, for
  // every 32-row tile, row i and the kept pairs of blocks 4h .. 4h+3; 2-bit positions at bits
  // [2e+1 : 2e].  The matrix-core copy is stored from here; the canonical values and metadata of
  // the four blocks are parked in the tile, over the 4M elements they came from, for phase 3.
  const int tiles = V / 32;
  // matrix-core copy: 64-row blocks of two 32-row tiles; tile `at` of this row block is tile
  // number r * tiles + at of the whole matrix
  const bool odd_tail = a.pa && tiles == 1 && (a.R & 1) && r == a.R - 1;   // V = 32: a last 64-row block with one real tile
  for (int item = tid; item < nks * 64; item += 256) {
    const int ks = item >> 6, lane = item & 63;
    const int i = lane & 31, h = lane >> 5;
    const int blk0 = ks * 8 + 4 * h;
    const uint4 kp4 = *(const uint4*)(keep + blk0);
    const unsigned kp[4] = {kp4.x, kp4.y, kp4.z, kp4.w};
    unsigned short ixs[4] = {0, 0, 0, 0};
    for (int at = 0; at < tiles; ++at) {
      const int v = at * 32 + i;
      unsigned short* trow = tile + (size_t)v * NCP + blk0 * M;
      unsigned q[4], ix = 0;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const unsigned short* tb = trow + g * M;
        const unsigned w0 = tb[kp[g] & 255u], w1 = tb[(kp[g] >> 8) & 255u], w2 = tb[(kp[g] >> 16) & 255u],
                       w3 = tb[kp[g] >> 24];
        unsigned nib;
        if constexpr (SCORED) {
          const float* sb = stile + (size_t)v * NCS + (blk0 + g) * M;
          nib = top2_of_4_s(__float_as_uint(sb[kp[g] & 255u]) & 0x7FFFFFFFu, __float_as_uint(sb[(kp[g] >> 8) & 255u]) & 0x7FFFFFFFu,
                            __float_as_uint(sb[(kp[g] >> 16) & 255u]) & 0x7FFFFFFFu, __float_as_uint(sb[kp[g] >> 24]) & 0x7FFFFFFFu);
          const unsigned w4[4] = {w0, w1, w2, w3};
          q[g] = w4[nib & 3] | (w4[nib >> 2] << 16);
        } else {
          nib = top2_of_4_f(w0, w1, w2, w3, q[g]);
        }
        ix |= nib << (4 * g);
      }
      ixs[at] = (unsigned short)ix;
      if (a.pa) {
        const int64_t gt = r * tiles + at;
        a.pa[(((gt >> 1) * a.S + s_begin + ks) * 2 + (gt & 1)) * 64 + lane] = make_uint4(q[0], q[1], q[2], q[3]);
      }
      // 8-byte aligned: blk0 is a multiple of 4
      *(uint2*)trow = make_uint2(q[0], q[1]);
      *(uint2*)(trow + 4) = make_uint2(q[2], q[3]);
      trow[8] = (unsigned short)ix;
    }
    if (a.pa) {
      if (tiles == 1) {
        a.pidx[(((r >> 1) * a.S + s_begin + ks) * 64 + lane) * 2 + (r & 1)] = ixs[0];
        if (odd_tail) {           // the missing second tile: values 0, positions (0, 1)
          a.pa[(((r >> 1) * a.S + s_begin + ks) * 2 + 1) * 64 + lane] = make_uint4(0, 0, 0, 0);
          a.pidx[(((r >> 1) * a.S + s_begin + ks) * 64 + lane) * 2 + 1] = (unsigned short)0x4444u;
        }
      } else {
        for (int sb = 0; sb < tiles / 2; ++sb)
          *(unsigned*)(a.pidx + (((r * (tiles / 2) + sb) * a.S + s_begin + ks) * 64 + lane) * 2) =
              (unsigned)ixs[2 * sb] | ((unsigned)ixs[2 * sb + 1] << 16);
      }
    }
  }
  __syncthreads();
  // phase 3: canonical values and metadata, a row's pieces stored by neighbouring lanes
  {
    const int64_t vrow_elems = 2 * a.B;
    const int64_t mrow = (a.B + 1) / 2;
    const bool v16 = (a.B & 3) == 0 && ((uintptr_t)a.values & 15) == 0;
    const int nq = nks * 2;                                  // groups of 4 blocks in this span
    const unsigned nq_inv = (65536u + nq - 1) / nq;
    for (int item = tid; item < V * nq; item += 256) {
      const int v = (int)(((unsigned)item * nq_inv) >> 16), qd = item - v * nq;   // item < 2^12, nq <= 16: exact
      const int blk0 = qd * 4;
      if (blk0 >= nbw) continue;
      const unsigned short* trow = tile + (size_t)v * NCP + blk0 * M;
      const uint2 lo = *(const uint2*)trow, hi = *(const uint2*)(trow + 4);
      const unsigned ix = trow[8];
      const int64_t row = r * V + v;
      unsigned short* vdst = a.values + row * vrow_elems + 2 * (b0 + blk0);
      if (v16 && blk0 + 4 <= nbw) {
        *(uint4*)vdst = make_uint4(lo.x, lo.y, hi.x, hi.y);
      } else {
        *(unsigned*)vdst = lo.x;
        if (blk0 + 1 < nbw) *(unsigned*)(vdst + 2) = lo.y;
        if (blk0 + 2 < nbw) *(unsigned*)(vdst + 4) = hi.x;
        if (blk0 + 3 < nbw) *(unsigned*)(vdst + 6) = hi.y;
      }
      // two blocks per byte; a block beyond the last real one leaves its nibble zero
      unsigned char* mdst = a.meta + row * mrow + ((b0 + blk0) >> 1);
      if (blk0 + 4 <= nbw) {
        const unsigned short two = (unsigned short)ix;
        __builtin_memcpy(mdst, &two, 2);
      } else {
        mdst[0] = (unsigned char)((ix & 15u) | (blk0 + 1 < nbw ? (ix & 0xF0u) : 0u));
        if (blk0 + 2 < nbw) mdst[1] = (unsigned char)(((ix >> 8) & 15u) | (blk0 + 3 < nbw ? ((ix >> 8) & 0xF0u) : 0u));
      }
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
      if (tiles == 1) {
        // two column tables per 64-row block, table r & 1 is this row block's
        a.pcol[((((r >> 1) * a.S + s_begin + ks) * 8 + h * 4 + kq) << 1) + (r & 1)] = o;
        if (odd_tail) {
          unsigned od = 0;
          for (int m = 0; m < 4; ++m) od |= (unsigned)((4 * (m >> 1) + 2 * h + (m & 1)) * M + kq) << (8 * m);
          a.pcol[((((r >> 1) * a.S + s_begin + ks) * 8 + h * 4 + kq) << 1) + 1] = od;
        }
      } else {
        for (int sb = 0; sb < tiles / 2; ++sb) a.pcol[((r * (tiles / 2) + sb) * a.S + s_begin + ks) * 8 + h * 4 + kq] = o;
      }
    }
  }
  // phase 4: optional dense 0-1 mask, from the positions parked in the tile
  if (a.mask) {
    for (int item = tid; item < V * NBW; item += 256) {
      const int v = item / NBW, b = item - v * NBW;
      if (b >= nbw) continue;
      const int64_t row = r * V + v;
      if (row >= a.out) continue;
      const unsigned ix = tile[(size_t)v * NCP + (b & ~3) * M + 8];
      const unsigned nib = (ix >> (4 * (b & 3))) & 15u;
      const unsigned kp = keep[b];
      const unsigned ca = (kp >> (8 * (nib & 3))) & 255u, cb = (kp >> (8 * (nib >> 2))) & 255u;
      const int64_t colb = (b0 + b) * M;
      for (int c = 0; c < M; ++c)
        if (colb + c < a.in) a.mask[row * a.in + colb + c] = (unsigned char)((unsigned)c == ca || (unsigned)c == cb);
    }
  }
}

// K steps per workgroup: 8 make every span of columns a whole number of 128-byte lines; fewer when
// the tile would not leave room for 3 workgroups per CU, or when the launch would be little more
// than one generation of workgroups on the 256 CUs (then shorter-lived workgroups overlap better),
// down to 1 when it would not even be one workgroup per CU (small matrices: the launch then lasts as
// long as one workgroup lives, and that is proportional to its tile).
static int prune_fast_ksw(const Dims& d) {
  int k = 8;
  while (k > 1 && (size_t)d.V * (k * 8 * d.M + 8) * 2 > 46 * 1024) k >>= 1;
  while (k > 4 && d.R * ((d.S + k - 1) / k) < 6 * 256) k >>= 1;
  while (k > 1 && d.R * ((d.S + k - 1) / k) < 256) k >>= 1;
  return k;
}

static size_t prune_fast_lds(int V, int M, int KSW, bool scored = false) {
  const size_t NC = (size_t)KSW * 8 * M, NBW = (size_t)KSW * 8;
  return (size_t)V * (NC + 4) * 2 + NC * 8 + NBW * 4 + (scored ? (size_t)V * (NC + 4) * 4 : 0);
}

bool prune_fast_applicable(const void* W, int64_t ldw, const Dims& d, const void* mask) {
  // ldw: a row's byte pitch is a 24-bit factor of a thread's 32-bit offset inside its workgroup's rows of W
  return d.M <= 16 && d.V % 32 == 0 && d.V <= 128 && d.in % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)W & 15) == 0 &&
         d.S <= 65535 && d.R <= 65535 && ldw < ((int64_t)1 << 23);
}

// Score-driven variant: the same kernel with the score tile next to the weight tile in LDS
bool prune_fast_scored_applicable(const void* W, int64_t ldw, const void* S, int64_t lds_s, const Dims& d) {
  return prune_fast_applicable(W, ldw, d, nullptr) && lds_s % 4 == 0 && ((uintptr_t)S & 15) == 0 &&
         prune_fast_lds(d.V, d.M, 1, true) <= 64 * 1024;
}

int launch_prune_fast_scored(const void* W, int64_t ldw, const void* S, int64_t lds_s, const Dims& d, void* values,
                             void* meta, void* colidx, void* mask, void* packed, hipStream_t st) {
  PruneFastArgs a{};
  a.W = (const unsigned short*)W; a.ldw = ldw; a.out = d.out; a.in = d.in; a.V = d.V; a.M = d.M;
  a.R = d.R; a.B = d.B; a.S = d.S;
  a.Sc = (const float*)S; a.lds_s = lds_s;
  int k = 8;
  while (k > 1 && prune_fast_lds(d.V, d.M, k, true) > 64 * 1024) k >>= 1;     // two workgroups per CU at least
  a.KSW = k;
  const int chunks = a.KSW * d.M;
  a.G = 256 / chunks < d.V ? 256 / chunks : d.V;
  a.values = (unsigned short*)values; a.meta = (unsigned char*)meta; a.colidx = (unsigned char*)colidx;
  a.mask = (unsigned char*)mask;
  if (packed) {
    const PackedLayout pl = packed_layout(d);
    char* p = (char*)packed;
    a.pa = (uint4*)(p + pl.pa_off); a.pidx = (unsigned short*)(p + pl.pidx_off); a.pcol = (unsigned*)(p + pl.pcol_off);
  }
  const size_t lds = prune_fast_lds(d.V, d.M, a.KSW, true);
  if (int rc_lds = allow_big_lds((const void*)prune_pack_kernel<true>, "hipFuncSetAttribute(prune_pack scored)")) return rc_lds;
  dim3 grid((unsigned)((d.S + a.KSW - 1) / a.KSW), (unsigned)d.R);
  hipLaunchKernelGGL(prune_pack_kernel<true>, grid, dim3(256), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "prune_pack_kernel<scored>"); return VNM_ERR_HIP; }
  return VNM_OK;
}

int launch_prune_fast(const void* W, int64_t ldw, const Dims& d, void* values, void* meta, void* colidx,
                      void* mask, void* packed, hipStream_t st) {
  PruneFastArgs a{};
  a.W = (const unsigned short*)W; a.ldw = ldw; a.out = d.out; a.in = d.in; a.V = d.V; a.M = d.M;
  a.R = d.R; a.B = d.B; a.S = d.S;
  a.KSW = prune_fast_ksw(d);
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
  const size_t lds = prune_fast_lds(d.V, d.M, a.KSW);
  if (int rc_lds = allow_big_lds((const void*)prune_pack_kernel<false>, "hipFuncSetAttribute(prune_pack)")) return rc_lds;
  // column spans along x: the workgroups that run together then read whole rows of W (every memory
  // channel in use) instead of one window of columns in many rows; on weights that come from HBM
  // 11008 x 4096 takes 62 us instead of 71, 4096 x 11008 66 instead of 71, 4096 x 4096 the same
  dim3 grid((unsigned)((d.S + a.KSW - 1) / a.KSW), (unsigned)d.R);
  hipLaunchKernelGGL(prune_pack_kernel<false>, grid, dim3(256), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "prune_pack_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

// ---------------------------------------------------------------- decompress
// One workgroup: V rows x KSW K steps (8 KSW column blocks).  The dense tile is assembled in LDS
// (zero fill, then two 2-byte scatters per (row, block), a thread taking 4 blocks of a row with one
// 16-byte load of values and one 2-byte load of metadata) and written out with 16-byte stores.
struct DecompArgs {
  const unsigned short* values; const unsigned char* meta; const unsigned char* colidx;
  int64_t out, in, B, S; int V, M, KSW, G;
  int spans_x;             // grid: column spans along x (else row blocks along x)
  unsigned short* Wd; int64_t ldw;
};

__global__ void __launch_bounds__(256) decompress_fast_kernel(const DecompArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int V = a.V, M = a.M;
  const int64_t r = a.spans_x ? blockIdx.y : blockIdx.x;
  const int64_t s_begin = (int64_t)(a.spans_x ? blockIdx.x : blockIdx.y) * a.KSW;
  const int nks = (int)((a.S - s_begin) < a.KSW ? (a.S - s_begin) : a.KSW);
  const int NC = a.KSW * 8 * M, NBW = a.KSW * 8;
  const int NCP = NC + 8;
  const int64_t b0 = s_begin * 8, c0 = b0 * M;
  const int nbw = (int)((a.B - b0) < nks * 8 ? (a.B - b0) : nks * 8);
  unsigned short* tile = (unsigned short*)smem;
  unsigned* keep = (unsigned*)(smem + (size_t)V * NCP * 2);
  const int tid = threadIdx.x;
  const int chunks = NC / 8, G = a.G;
  const int g = tid / chunks, ch = tid - g * chunks;
  if (g < G)
    for (int v = g; v < V; v += G) *(uint4*)(tile + (size_t)v * NCP + ch * 8) = make_uint4(0, 0, 0, 0);
  for (int b = tid; b < nbw; b += 256) keep[b] = *(const unsigned*)(a.colidx + (r * a.B + b0 + b) * 4);
  __syncthreads();
  {
    const int64_t vrow_elems = 2 * a.B, mrow = (a.B + 1) / 2;
    const bool v16 = (a.B & 3) == 0 && ((uintptr_t)a.values & 15) == 0;
    const int nq = nks * 2;
    const unsigned nq_inv = (65536u + nq - 1) / nq;
    for (int item = tid; item < V * nq; item += 256) {
      const int v = (int)(((unsigned)item * nq_inv) >> 16), qd = item - v * nq;   // item < 2^12, nq <= 16: exact
      const int blk0 = qd * 4;
      const int64_t row = r * V + v;
      if (blk0 >= nbw || row >= a.out) continue;
      const unsigned short* vsrc = a.values + row * vrow_elems + 2 * (b0 + blk0);
      const unsigned char* msrc = a.meta + row * mrow + ((b0 + blk0) >> 1);
      unsigned q[4] = {0, 0, 0, 0}, ix;
      if (blk0 + 4 <= nbw) {
        if (v16) { const uint4 t = *(const uint4*)vsrc; q[0] = t.x; q[1] = t.y; q[2] = t.z; q[3] = t.w; }
        else { for (int e = 0; e < 4; ++e) q[e] = *(const unsigned*)(vsrc + 2 * e); }
        unsigned short two;
        __builtin_memcpy(&two, msrc, 2);
        ix = two;
      } else {
        for (int e = 0; e < 4; ++e) if (blk0 + e < nbw) q[e] = *(const unsigned*)(vsrc + 2 * e);
        ix = msrc[0];
        if (blk0 + 2 < nbw) ix |= (unsigned)msrc[1] << 8;
      }
      unsigned short* trow = tile + (size_t)v * NCP + blk0 * M;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (blk0 + e < nbw) {
          const unsigned nib = (ix >> (4 * e)) & 15u, kp = keep[blk0 + e];
          const unsigned ca = min((kp >> (8 * (nib & 3))) & 255u, (unsigned)M - 1u);
          const unsigned cb = min((kp >> (8 * (nib >> 2))) & 255u, (unsigned)M - 1u);
          trow[e * M + ca] = (unsigned short)(q[e] & 0xFFFFu);
          trow[e * M + cb] = (unsigned short)(q[e] >> 16);
        }
      }
    }
  }
  __syncthreads();
  if (g < G) {
    const int64_t col = c0 + ch * 8;
    if (col < a.in)
      for (int v = g; v < V; v += G) {
        const int64_t row = r * V + v;
        if (row < a.out) *(uint4*)(a.Wd + row * a.ldw + col) = *(const uint4*)(tile + (size_t)v * NCP + ch * 8);
      }
  }
}

bool decompress_fast_applicable(const void* W_out, int64_t ldw, const Dims& d) {
  return d.M <= 16 && d.V <= 128 && d.in % 8 == 0 && ldw % 8 == 0 && ((uintptr_t)W_out & 15) == 0 && d.S <= 65535 &&
         d.R <= 65535;
}

int launch_decompress_fast(const void* values, const void* meta, const void* colidx, const Dims& d,
                           void* W_out, int64_t ldw, hipStream_t st) {
  DecompArgs a;
  a.values = (const unsigned short*)values; a.meta = (const unsigned char*)meta; a.colidx = (const unsigned char*)colidx;
  a.out = d.out; a.in = d.in; a.B = d.B; a.S = d.S; a.V = d.V; a.M = d.M;
  a.KSW = prune_fast_ksw(d);
  const int chunks = a.KSW * d.M;
  a.G = 256 / chunks < d.V ? 256 / chunks : d.V;
  a.Wd = (unsigned short*)W_out; a.ldw = ldw;
  const size_t lds = (size_t)d.V * (a.KSW * 8 * d.M + 8) * 2 + (size_t)a.KSW * 8 * 4;
  if (int rc_lds = allow_big_lds((const void*)decompress_fast_kernel, "hipFuncSetAttribute(decompress_fast)")) return rc_lds;
  // Workgroups that run together should cover whole rows of W' (all column spans of a few row blocks:
  // every memory channel is in use) rather than one window of columns in many rows -- unless a span is
  // not a whole number of 128-byte lines: then neighbouring spans share lines, and writing the two
  // parts of a line at the same time from different XCDs costs more than the channels bring
  // (4096 x 4096, 64:2:5: 12.3 us with row blocks along x, 14.7 us with spans along x; 11008 x 4096,
  // whole lines: 33.3 against 29.8 us).
  const unsigned n_spans = (unsigned)((d.S + a.KSW - 1) / a.KSW);
  a.spans_x = (a.KSW * 8 * d.M * 2) % 128 == 0;
  dim3 grid(a.spans_x ? n_spans : (unsigned)d.R, a.spans_x ? (unsigned)d.R : n_spans);
  hipLaunchKernelGGL(decompress_fast_kernel, grid, dim3(256), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "decompress_fast_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
