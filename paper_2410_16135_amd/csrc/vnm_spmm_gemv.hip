// vnm_spmm for at most 4 tokens (decode at batch 1..4): the product as a stream of the packed weight
// through the vector ALUs, without the matrix cores.
//
// With one to four tokens the work is bound by the bytes of the compressed weight (Section 3,
// "Acceleration of V:N:M sparsity": the compressed weight is what has to be read), and a matrix
// instruction would spend 32 token columns on them: every lane would gather 16 halfwords of X per
// instruction pair for tokens that do not exist.  Here a lane keeps the role it has in the packed
// copy -- row i of a 32-row tile, half h of a K step, i.e. the two kept values of 4 column blocks per
// step -- and multiplies them itself:
//   * the 4 kept columns of a block are the same for all rows of the tile, so the 32 halfwords of X
//     that a (tile, K step, token) needs are fetched once per wave (lane j fetches entry j from the
//     copy of X in LDS, at the offset the packed column table gives) and left in a 64-byte strip of
//     LDS in the order the lanes use them; a lane reads its half of the strip back with two 16-byte
//     reads that are the same address for 32 lanes (broadcast);
//   * the 2-bit positions of a lane's two values in a block become one byte selector, and one
//     V_PERM_B32 picks the two matching halfwords of X out of the block's four; one V_DOT2_F32_F16
//     adds the two products to the lane's fp32 sum.
// One workgroup owns one 32-row tile and all of K; each of its waves takes a contiguous range of K steps
// with a ring of steps of weights requested ahead, and the waves add their sums through LDS at the end.
#include "vnm_internal.h"

namespace vnm {

typedef _Float16 gv_h2 __attribute__((ext_vector_type(2)));

// All operands are addressed with 32-bit byte offsets from their base pointers (the launcher checks
// that they fit): one address register per load instead of two.
struct GemvArgs {
  const unsigned char* X; int64_t T, ldx, in;
  const unsigned char* pa; const unsigned char* pidx; const unsigned char* pcol;
  int64_t out, S;
  int M;
  void* Y; int64_t ldy; int y_fp32;
  const _Float16* bias; const int* perm_out;     // fused epilogue (null = none), as in the few-token kernels
};

// NTOK: token rows computed (1, 2 or 4; rows beyond T count as zero and are not stored).
// DUAL: the 64-row block carries one column table per 32-row tile (V = 32 patterns).
// WAVES: waves per workgroup; RING: K steps of weights a wave requests ahead.
template <int NTOK, bool DUAL, int WAVES, int RING>
__global__ void __launch_bounds__(64 * WAVES) spmm_gemv_kernel(const GemvArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NT = DUAL ? 2 : 1;
  constexpr int THREADS = 64 * WAVES;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const unsigned rp = blockIdx.x >> 1;             // 64-row block of the packed copy
  const unsigned at = blockIdx.x & 1;              // its 32-row tile
  const unsigned S = (unsigned)a.S;
  const int M = a.M;
  const int in = (int)a.in;
  const int xpitch = in * 2 + 128;                 // bytes per token row of X in LDS
  unsigned char* xlds = smem;
  // this wave's strips: [ring slot][token][32 halfwords]
  unsigned char* xg = smem + (size_t)NTOK * xpitch + (size_t)wave * (RING * NTOK * 64);
  float* red = (float*)(smem + (size_t)NTOK * xpitch + (size_t)WAVES * RING * NTOK * 64);

  // entry j of a strip is kept column kq of block 4 hj + g of the step; its offset inside the step's
  // 8 M raw columns is byte 2 hj + (g & 1) of dword ((g >> 1) * 4 + kq) (per table) of the column table
  const int j = lane & 31, hj = j >> 4, gj = (j >> 2) & 3, kqj = j & 3;
  const int pcb_off = ((((gj >> 1) * 4 + kqj) * NT + (DUAL ? at : 0)) << 2) + 2 * hj + (gj & 1);
  const int tokhalf = lane >> 5;                   // gather: lanes 0..31 take tokens 0, 2; lanes 32..63 tokens 1, 3
  const int hA = lane >> 5;                        // multiply: half of the K step

  struct Slot { uint4 w; unsigned idx, pcb; };
  // this wave's K steps: a contiguous range
  const unsigned per = (S + WAVES - 1) / WAVES;
  const unsigned s0 = wave * per < S ? wave * per : S;
  const unsigned s1 = s0 + per < S ? s0 + per : S;
  // Loads beyond the range are still issued (the count of loads in flight is the same on every path),
  // but every lane then reads lane 0's operand of step 0 of the tile: one cache line, not eight.
  auto load_pcb = [&](Slot& o, unsigned s) {
    s = s < s1 ? s : 0;
    o.pcb = a.pcol[(rp * S + s) * (32u * NT) + pcb_off];
  };
  auto load_w = [&](Slot& o, unsigned s) {
    const unsigned l = s < s1 ? lane : 0;
    s = s < s1 ? s : 0;
    const unsigned rs = rp * S + s;
    o.idx = *(const unsigned short*)(a.pidx + (((rs * 64 + l) * 2 + at) * 2u));
    o.w = *(const uint4*)(a.pa + (((rs * 2 + at) * 64 + l) * 16u));
  };
  auto load = [&](Slot& o, unsigned s) { load_pcb(o, s); load_w(o, s); };
  Slot ring[RING];

  // X -> LDS, token rows as they are, in 16-byte pieces (pieces tid, tid + THREADS, ... of every token
  // row).  The first piece of every row is requested before the weights (loads return in order, and X
  // comes from L2 while the weights come from HBM) and parked while the weights travel; rows longer
  // than 8 * THREADS halfwords fetch the rest behind the weights.
  {
    const int cpr = in / 8;                        // pieces per row
    const unsigned ldxb = (unsigned)a.ldx * 2u;
    const int t_last = (a.T < NTOK ? (int)a.T : NTOK) - 1;
    uint4 xw[NTOK];
    const unsigned c0 = tid < cpr ? tid : cpr - 1;   // clamped; dropped below
#pragma unroll
    for (int t = 0; t < NTOK; ++t) {
      const unsigned tt = t < t_last ? t : t_last;
      xw[t] = *(const uint4*)(a.X + (tt * ldxb + c0 * 16u));
    }
    // every wave's requests for X are queued before any wave's requests for weights: the unit's memory
    // pipeline serves them in order, and the barrier below cannot fall before the last piece of X
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < RING; ++i) load_pcb(ring[i], s0 + i);
#pragma unroll
    for (int i = 0; i < RING; ++i) load_w(ring[i], s0 + i);
#pragma unroll
    for (int t = 0; t < NTOK; ++t) {
      const uint4 v = xw[t];
      if (t <= t_last && tid < cpr) *(uint4*)(xlds + (size_t)t * xpitch + tid * 16) = v;
    }
    for (int c = tid + THREADS; c < cpr; c += THREADS)
      for (int t = 0; t <= t_last; ++t)
        *(uint4*)(xlds + (size_t)t * xpitch + c * 16) = *(const uint4*)(a.X + ((unsigned)t * ldxb + (unsigned)c * 16u));
  }
  __syncthreads();

  float acc[NTOK];
#pragma unroll
  for (int t = 0; t < NTOK; ++t) acc[t] = 0.f;

  // The 32 halfwords of X that the steps of a round need, per token, into the round's strips: all reads
  // first, then all stores (two LDS round trips per round).  Branch-free: a column beyond `in` or a
  // token beyond T reads X[0][0] and stores zero; with one token both halves of the wave do the same.
  // A slot beyond the wave's range holds step 0's column table: its strip is filled and never used.
  constexpr int NIT = (NTOK + 1) / 2;
  const int tg0 = tokhalf < NTOK ? tokhalf : NTOK - 1;          // token of this lane in gather pass 0
  auto gather_round = [&](unsigned sb) {
    unsigned short v[RING][NIT];
#pragma unroll
    for (int i = 0; i < RING; ++i) {
      const unsigned s = sb + i < s1 ? sb + i : 0;
      const int col = (int)s * 8 * M + (int)ring[i].pcb;
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int t = it == 0 ? tg0 : 2 * it + tokhalf;
        const bool ok = t < a.T && col < in;
        const unsigned short x = *(const unsigned short*)(xlds + (ok ? t * xpitch + col * 2 : 0));
        v[i][it] = ok ? x : (unsigned short)0;
      }
    }
#pragma unroll
    for (int i = 0; i < RING; ++i)
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int t = it == 0 ? tg0 : 2 * it + tokhalf;
        *(unsigned short*)(xg + (i * NTOK + t) * 64 + j * 2) = v[i][it];
      }
  };
  auto multiply = [&](const Slot& o, int slot) {
    const unsigned ix = o.idx;
    unsigned sel[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // positions p0 (bits 0..1) and p1 (bits 2..3) of the block's nibble -> byte selector
      // (2 p0, 2 p0 + 1, 2 p1, 2 p1 + 1): p0 | p1 << 16, times 0x0202, plus 0x01000100
      const unsigned y = ix >> (4 * g);
      sel[g] = ((y | (y << 14)) & 0x00030003u) * 0x0202u + 0x01000100u;
    }
    const unsigned wv[4] = {o.w.x, o.w.y, o.w.z, o.w.w};
#pragma unroll
    for (int t = 0; t < NTOK; ++t) {
      const unsigned char* strip = xg + (slot * NTOK + t) * 64 + hA * 32;
      const uint4 x0 = *(const uint4*)strip, x1 = *(const uint4*)(strip + 16);
      const unsigned xd[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const unsigned xs = __builtin_amdgcn_perm(xd[2 * g + 1], xd[2 * g], sel[g]);
        // both products exact in fp32, added to the sum in fp32 (V_DOT2_F32_F16)
        acc[t] = __builtin_amdgcn_fdot2(__builtin_bit_cast(gv_h2, wv[g]), __builtin_bit_cast(gv_h2, xs), acc[t], false);
      }
    }
  };

  for (unsigned sb = s0; sb < s1; sb += RING) {
    gather_round(sb);
    // the strips are read back by other lanes of the same wave: LDS executes a wave's accesses in
    // order; the fences keep the compiler from moving the reads in front of the stores
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (sb + RING < s1) {
      // another round follows: every slot is refilled as soon as it has been multiplied
#pragma unroll
      for (int i = 0; i < RING; ++i) {
        multiply(ring[i], i);
        load(ring[i], sb + RING + i);
      }
    } else {
      // the last round requests nothing
#pragma unroll
      for (int i = 0; i < RING; ++i)
        if (sb + i < s1) multiply(ring[i], i);
    }
    __builtin_amdgcn_wave_barrier();               // the next round's stores to the strips stay behind these reads
  }

#pragma unroll
  for (int t = 0; t < NTOK; ++t) red[(wave * NTOK + t) * 64 + lane] = acc[t];
  __syncthreads();
  for (int e = tid; e < 32 * NTOK; e += THREADS) {
    const int tok = e >> 5, i = e & 31;
    const int64_t o = (int64_t)rp * 64 + at * 32 + i;
    if (tok < a.T && o < a.out) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        sum += red[(w * NTOK + tok) * 64 + i];
        sum += red[(w * NTOK + tok) * 64 + 32 + i];
      }
      if (a.bias) sum += (float)a.bias[o];
      const int64_t dst = a.perm_out ? (int64_t)a.perm_out[o] : o;          // Eq. 6, P_o^T
      if (dst < 0 || dst >= a.out) continue;
      if (a.y_fp32) ((float*)a.Y)[tok * a.ldy + dst] = sum;
      else ((_Float16*)a.Y)[tok * a.ldy + dst] = (_Float16)sum;
    }
  }
}

int64_t gemv_max_tokens() { return 4; }

static size_t gemv_lds(int ntok, int64_t in, int waves, int ring) {
  return (size_t)ntok * ((size_t)in * 2 + 128) + (size_t)waves * ring * ntok * 64 + (size_t)waves * ntok * 64 * 4;
}

static int gemv_ntok(int64_t T) { return T <= 1 ? 1 : (T <= 2 ? 2 : 4); }

// Workgroup shape, from timings of the Llama-2-7B layer shapes at 64:2:5 with the weights coming from
// HBM.  More tiles than compute units: 8 waves, so that several workgroups share a unit and one's
// start-up (X, the first weights) overlaps the others' streaming; otherwise 16 waves.  A ring of 2 steps
// per wave is enough: the stream is kept going by the 16 to 32 waves of a unit, and deeper rings
// measured slower (ring 2 / 4 / 8, 4096 x 4096, one token: 7.0 / 7.2 / 8.1 us).
constexpr int kGvRing = 2;
static int gemv_waves(const Dims& d) { return 2 * packed_row_blocks(d) > 256 ? 8 : 16; }

bool spmm_gemv_applicable(int64_t T, int64_t ldx, const Dims& d) {
  if (T < 1 || T > gemv_max_tokens() || !has_packed(d.V, d.M) || d.in % 8) return false;
  // 32-bit byte offsets: rows of X, the packed copy, raw column numbers
  if (T * ldx * 2 > 0x7FFFFFFF || packed_layout(d).total > 0x7FFFFFFF || d.S * 8 * d.M + 128 > 0x7FFFFFFF) return false;
  if (2 * packed_row_blocks(d) > 0x7FFFFFFF) return false;
  // Three and four tokens: only where the tiles leave compute units idle and K is short.  Otherwise the
  // vector ALUs become the limit and the matrix-core few-token kernel is faster (device time per call
  // at four tokens, 64:2:5, weights from HBM, this kernel / that one: 4096 x 4096, 103 K steps, 8.0 / 10.6 us;
  // 11008 x 4096, 344 tiles, 13.2 / 12.7 us; 4096 x 11008, 276 K steps, 16.4 / 13.8 us)
  if (T > 2 && (2 * packed_row_blocks(d) > 256 || d.S > 224)) return false;
  return gemv_lds(gemv_ntok(T), d.in, gemv_waves(d), kGvRing) <= 150 * 1024;
}

template <int NTOK, bool DUAL, int WAVES>
static int launch_gemv_cfg(const GemvArgs& a, int64_t Rp, hipStream_t st) {
  auto kern = spmm_gemv_kernel<NTOK, DUAL, WAVES, kGvRing>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(spmm_gemv)")) return rc_lds;
  hipLaunchKernelGGL(kern, dim3((unsigned)(2 * Rp)), dim3(64 * WAVES), gemv_lds(NTOK, a.in, WAVES, kGvRing), st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_gemv_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

template <int NTOK, bool DUAL>
static int launch_gemv_shape(const GemvArgs& a, const Dims& d, hipStream_t st) {
  const int64_t Rp = packed_row_blocks(d);
  return gemv_waves(d) == 8 ? launch_gemv_cfg<NTOK, DUAL, 8>(a, Rp, st) : launch_gemv_cfg<NTOK, DUAL, 16>(a, Rp, st);
}

// X: 16-byte aligned, ldx a multiple of 8 (what spmm_smfmac_applicable checks); spmm_gemv_applicable(T, ldx, d) holds
int launch_spmm_gemv(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                     void* Y, int64_t ldy, int y_dtype, const Fused& f, hipStream_t st) {
  const PackedLayout pl = packed_layout(d);
  const unsigned char* p = (const unsigned char*)packed;
  GemvArgs a{};
  a.X = (const unsigned char*)X; a.T = T; a.ldx = ldx; a.in = d.in;
  a.pa = p + pl.pa_off; a.pidx = p + pl.pidx_off; a.pcol = p + pl.pcol_off;
  a.out = d.out; a.S = d.S; a.M = d.M;
  a.Y = Y; a.ldy = ldy; a.y_fp32 = y_dtype;
  a.bias = f.bias; a.perm_out = f.perm_out;
  const bool dual = packed_tables(d.V) == 2;
  switch (gemv_ntok(T)) {
    case 1: return dual ? launch_gemv_shape<1, true>(a, d, st) : launch_gemv_shape<1, false>(a, d, st);
    case 2: return dual ? launch_gemv_shape<2, true>(a, d, st) : launch_gemv_shape<2, false>(a, d, st);
    default: return dual ? launch_gemv_shape<4, true>(a, d, st) : launch_gemv_shape<4, false>(a, d, st);
  }
}

}  // namespace vnm
