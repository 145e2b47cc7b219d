// vnm_spmm without a staging pass, for products whose slice of X fits the LDS of a CU: short K at any
// token count (the DeiT-shaped layers of Section 5.1), and up to 256 tokens at any K (the batch sizes
// of Appendix E) with K cut into parts.
//
// A workgroup owns 64 tokens and a range of K steps.  It reads its slice of X straight from the
// caller's matrix, once, and turns it around on the way into LDS: [raw input column][token], the
// order the transposing LDS read of the matrix-core kernel wants (vnm_spmm_smfmac.hip: one
// ds_read_b64_tr_b16 fetches, for 16 tokens, the 4 kept columns of a column block, the rows chosen
// per lane from the packed column table).  After one barrier nothing is written to LDS any more:
// the K loop has no barrier and no copies, only the weight stream -- every wave keeps a ring of A
// operands requested ahead of the one it multiplies -- and the gathers.  Two shapes of the same
// kernel:
//   * row mode (KW = 1): the 8 waves take the row blocks of the workgroup's range in turn, a
//     64-row block each, over the whole K range; results go to Y straight from the accumulators.
//   * K mode (KW = 8 / RBW > 1): RBW row blocks per workgroup, the K steps of each dealt to KW waves,
//     whose accumulators are added up through LDS (the slice of X is dead by then).  For few tokens,
//     where there are not enough (token tile, row block) pairs to occupy the chip otherwise.
// K parts (gridDim.z > 1, K mode only) leave fp32 partial products in the caller's scratch; the
// workgroup that arrives last at a (token tile, row group) adds them up in a fixed order and stores Y,
// so the result does not depend on the arrival order and no second launch is needed.  Arrivals are
// counted in the scratch as well, in 64-bit slots tagged with a number that is unique to the call:
// a slot whose tag is not the call's counts as zero, so the scratch needs no clearing.
#include <atomic>
#include <chrono>
#include <random>
#include "vnm_internal.h"

namespace vnm {

typedef _Float16 rs_h8 __attribute__((ext_vector_type(8)));
typedef _Float16 rs_h16 __attribute__((ext_vector_type(16)));
typedef _Float16 rs_h4 __attribute__((ext_vector_type(4)));
typedef float rs_f16 __attribute__((ext_vector_type(16)));
typedef float rs_f4 __attribute__((ext_vector_type(4)));
typedef short rs_s4 __attribute__((__vector_size__(4 * sizeof(short))));
#define VNM_RS_LDS(T) __attribute__((address_space(3))) T*

constexpr int kResTok = 64;            // tokens per workgroup
constexpr int kResWaves = 8;
constexpr int kResRing = 6;            // A operands a wave keeps in flight
constexpr int kResRedPitch = 65;       // floats per token row of the in-workgroup reduction
constexpr size_t kResLdsMax = 150 * 1024;
constexpr int kResEpPitch = 144;       // row mode, fp16 epilogue: bytes per token row of a wave's strip
constexpr int kResEpBytes = 32 * kResEpPitch;

struct ResArgs {
  const unsigned short* X; int64_t T, ldx, in;
  const uint4* pa; const unsigned* pidx; const unsigned* pcol;
  int64_t out, R, S;                   // R: 64-row blocks of the packed copy
  int M, pitch;                        // pitch: bytes between image rows in LDS (a multiple of 8)
  int nsz;                             // K steps per K part
  int rb_per;                          // row blocks per workgroup (a multiple of RBW)
  void* Y; int64_t ldy; int y_fp32, vec_store;
  int wide_store;                      // row mode: fp16 Y with 16-byte stores through the LDS strips at ep_off
  unsigned ep_off;
  float* part;                         // [parts][T][out] fp32 when gridDim.z > 1
  unsigned long long* arrivals;        // [token tiles][R] slots
  unsigned long long tag;              // this call's tag (40 bits, never 0)
  const _Float16* bias; const int* perm_out;
};

// One arrival at `slot`; returns the number of arrivals of this call including this one.
__device__ inline unsigned arrive(unsigned long long* slot, unsigned long long tag) {
  unsigned long long old = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (;;) {
    const unsigned long long want = (old >> 24) == tag ? old + 1 : ((tag << 24) | 1ull);
    if (__hip_atomic_compare_exchange_strong(slot, &old, want, __ATOMIC_ACQ_REL, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT))
      return (unsigned)(want & 0xFFFFFFull);
  }
}

// DUAL: the 64-row block carries one column table per 32-row tile (V = 32 patterns).
// RBW: row blocks a workgroup works on at a time; KW = 8 / RBW waves share the K steps of each.
// ROWS: row mode (RBW = 8) instead of K mode.
template <bool DUAL, int RBW, bool ROWS>
__global__ void __launch_bounds__(64 * kResWaves) spmm_resident_kernel(const ResArgs a) {
  static_assert(!ROWS || RBW == 8, "row mode gives every wave a row block of its own");
  constexpr int KW = kResWaves / RBW;
  constexpr int NT = DUAL ? 2 : 1;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int M = a.M, P = a.pitch;
  const int64_t tile = blockIdx.x, t0 = tile * kResTok;
  const int64_t s_lo = (int64_t)blockIdx.z * a.nsz;
  const int64_t s_hi = s_lo + a.nsz < a.S ? s_lo + a.nsz : a.S;
  const int nst = (int)(s_hi - s_lo);                       // K steps of this workgroup
  const int64_t col0 = s_lo * 8 * M;
  const int CH = nst * M;                                   // 16-byte chunks per token

  // ---- the slice of X -> LDS, transposed.  Eight lanes share a token (a whole 128-byte line of its
  // row per load), a wave-wide load covers 8 tokens x 8 chunks; every lane then stores its 8 columns
  // to 8 image rows, two bytes each.  Rows beyond T and columns beyond `in` become zero (the packed
  // copy holds zero weights there, and zero times whatever else LDS held could be NaN).
  {
    const int tsub = lane >> 3, csub = lane & 7;
    constexpr int NB = 6;                                    // loads in flight per thread
    const int n_cg = (CH + 7) / 8;                           // chunk groups of 8
    // unit u = (chunk group, token group of 8): wave w takes units w, w + 8, ...
    const int units = n_cg * (kResTok / 8);
    for (int u0 = wave; u0 < units; u0 += kResWaves * NB) {
      uint4 xw[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int u = u0 + kResWaves * i;
        const int tok = (u & 7) * 8 + tsub, ch = (u >> 3) * 8 + csub;
        const bool ok = u < units && ch < CH && t0 + tok < a.T && col0 + ch * 8 < a.in;
        const unsigned short* src = ok ? a.X + (t0 + tok) * a.ldx + col0 + ch * 8 : a.X;
        xw[i] = *(const uint4*)src;
      }
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int u = u0 + kResWaves * i;
        const int tok = (u & 7) * 8 + tsub, ch = (u >> 3) * 8 + csub;
        if (u < units && ch < CH) {
          const bool ok = t0 + tok < a.T && col0 + ch * 8 < a.in;
          const uint4 v = ok ? xw[i] : make_uint4(0, 0, 0, 0);
          unsigned char* d = smem + (size_t)(ch * 8) * P + tok * 2;
          const unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            *(unsigned short*)(d + (size_t)(2 * e) * P) = (unsigned short)(w4[e] & 0xFFFFu);
            *(unsigned short*)(d + (size_t)(2 * e + 1) * P) = (unsigned short)(w4[e] >> 16);
          }
        }
      }
    }
  }

  // ---- roles
  const int wr = wave % RBW, wk = wave / RBW;               // row block within the group, K slice
  const int hB = lane >> 5, tg = (lane >> 4) & 1, kq = (lane & 15) >> 2, q = lane & 3;
  const unsigned tokoff = (unsigned)((tg * 16 + q * 4) * 2);
  const int64_t rb_lo = (int64_t)blockIdx.y * a.rb_per;
  const int64_t rb_hi = rb_lo + a.rb_per < a.R ? rb_lo + a.rb_per : a.R;
  const int ngroups = (int)((rb_hi - rb_lo + RBW - 1) / RBW);
  const int nmine = nst > wk ? (nst - wk + KW - 1) / KW : 0;          // K steps of this wave per row block
  // A wave's work is a list of items, row group by row group; a group's nmine steps are padded to a
  // multiple of the ring size, so that item n always sits in ring slot n % kResRing (slots are
  // registers, their index must be a constant).  Padding items are loaded like real ones (from a
  // valid address) and never multiplied.
  const int nmine_p = (nmine + kResRing - 1) / kResRing * kResRing;

  struct AOp { uint4 w[2]; unsigned idx; unsigned pc[NT]; };
  // operand of step number `i` (of this wave) of row group `g`; every load is unconditional, indices
  // beyond the ends are clamped to valid ones
  auto load_a = [&](AOp& o, int g, int i) {
    int64_t rb = rb_lo + (int64_t)g * RBW + wr;
    rb = rb < a.R ? rb : a.R - 1;
    const int64_t s = s_lo + wk + (int64_t)KW * i;
    const int64_t rs = rb * a.S + (s < a.S ? s : a.S - 1);
    o.w[0] = a.pa[(rs * 2) * 64 + lane];
    o.w[1] = a.pa[(rs * 2 + 1) * 64 + lane];
    o.idx = a.pidx[rs * 64 + lane];
#pragma unroll
    for (int t = 0; t < NT; ++t) o.pc[t] = a.pcol[(rs * 8 + hB * 4 + kq) * NT + t];
  };
  AOp ring[kResRing];
#pragma unroll
  for (int i = 0; i < kResRing; ++i) load_a(ring[i], 0, i);
  __syncthreads();                                          // the image is complete

  rs_f16 acc[2][2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[t][j][k] = 0.f;
  };
  zero_acc();

  const unsigned lds0 = (unsigned)(size_t)(VNM_RS_LDS(unsigned char))smem;
  auto compute = [&](const AOp& o, int ls) {                // ls: K step relative to s_lo
    const int ix = (int)o.idx;
    const unsigned base = lds0 + (unsigned)(ls * 8 * M) * (unsigned)P + tokoff;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      unsigned row[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) row[m] = base + ((o.pc[t] >> (8 * m)) & 255u) * (unsigned)P;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        rs_s4 b4[4];
#pragma unroll
        for (int m = 0; m < 4; ++m)
          b4[m] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((VNM_RS_LDS(rs_s4))(size_t)(row[m] + (unsigned)(j * 64)));
        typedef short rs_s16 __attribute__((__vector_size__(16 * sizeof(short))));
        rs_s16 bs;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
          for (int e = 0; e < 4; ++e) bs[4 * m + e] = b4[m][e];
        const rs_h16 bv = __builtin_bit_cast(rs_h16, bs);
        if (!DUAL || t == 0)
          acc[0][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(rs_h8, o.w[0]), bv, acc[0][j], ix, 0, 0);
        if (!DUAL || t == 1)
          acc[1][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(rs_h8, o.w[1]), bv, acc[1][j], ix, 0, 1);
      }
    }
  };

  const int tokl = lane & 31;
  const bool split = gridDim.z > 1;
  // Accumulator element 4 jq + e of tile (t, j) is channel rb * 64 + t * 32 + 8 jq + 4 hB + e of token
  // t0 + 32 j + tokl.  Row mode: straight to Y.
  auto store_rows = [&](int64_t rb) {
    if (a.wide_store && (rb + 1) * 64 <= a.out) {
      // fp16 Y that takes 16-byte stores: a lane holds 4 consecutive channels of one token per
      // register quad, so straight stores would put 8 bytes into each of 32 rows of Y per
      // instruction.  The wave turns its tile around in a private strip of LDS instead, 32 tokens at
      // a time ([token][64 channels], 144 bytes apart), and stores whole 128-byte runs of 8 rows.
      unsigned char* ep = smem + a.ep_off + (size_t)wave * kResEpBytes;
      _Float16* Yh = (_Float16*)a.Y;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int jq = 0; jq < 4; ++jq) {
            const int ch = t * 32 + 8 * jq + 4 * hB;
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
            if (a.bias) {
#pragma unroll
              for (int e = 0; e < 4; ++e) bv[e] = (float)a.bias[rb * 64 + ch + e];
            }
            rs_h4 pk = {(_Float16)(acc[t][j][4 * jq] + bv[0]), (_Float16)(acc[t][j][4 * jq + 1] + bv[1]),
                        (_Float16)(acc[t][j][4 * jq + 2] + bv[2]), (_Float16)(acc[t][j][4 * jq + 3] + bv[3])};
            *(rs_h4*)(ep + (size_t)tokl * kResEpPitch + ch * 2) = pk;
          }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int tk = it * 8 + (lane >> 3), c8 = lane & 7;
          const uint4 v = *(const uint4*)(ep + (size_t)tk * kResEpPitch + c8 * 16);
          const int64_t tok = t0 + j * 32 + tk;
          if (tok < a.T) *(uint4*)(Yh + tok * a.ldy + rb * 64 + c8 * 8) = v;
        }
      }
      return;
    }
    if (!a.perm_out && a.vec_store && (rb + 1) * 64 <= a.out) {
      // all 64 channels exist and Y takes 4-wide stores: no per-element tests
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int jq = 0; jq < 4; ++jq) {
          const int64_t o = rb * 64 + t * 32 + 8 * jq + 4 * hB;
          float bv[4] = {0.f, 0.f, 0.f, 0.f};
          if (a.bias) {
#pragma unroll
            for (int e = 0; e < 4; ++e) bv[e] = (float)a.bias[o + e];
          }
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const int64_t tok = t0 + j * 32 + tokl;
            if (tok < a.T) {
              if (a.y_fp32) {
                rs_f4 pk = {acc[t][j][4 * jq] + bv[0], acc[t][j][4 * jq + 1] + bv[1], acc[t][j][4 * jq + 2] + bv[2],
                            acc[t][j][4 * jq + 3] + bv[3]};
                *(rs_f4*)((float*)a.Y + tok * a.ldy + o) = pk;
              } else {
                rs_h4 pk = {(_Float16)(acc[t][j][4 * jq] + bv[0]), (_Float16)(acc[t][j][4 * jq + 1] + bv[1]),
                            (_Float16)(acc[t][j][4 * jq + 2] + bv[2]), (_Float16)(acc[t][j][4 * jq + 3] + bv[3])};
                *(rs_h4*)((_Float16*)a.Y + tok * a.ldy + o) = pk;
              }
            }
          }
        }
      return;
    }
    // ragged last row block, unaligned Y, or an output permutation: element by element
#pragma unroll
    for (int tj = 0; tj < 8; ++tj) {
      const int t = tj >> 2, jq = tj & 3;
      const int64_t o = rb * 64 + t * 32 + 8 * jq + 4 * hB;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (o + e >= a.out) continue;
        const float bvv = a.bias ? (float)a.bias[o + e] : 0.f;
        const int64_t dst = a.perm_out ? (int64_t)a.perm_out[o + e] : o + e;      // Eq. 6, P_o^T
        if (dst < 0 || dst >= a.out) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int64_t tok = t0 + j * 32 + tokl;
          if (tok >= a.T) continue;
          const float v = acc[t][j][4 * jq + e] + bvv;
          if (a.y_fp32) ((float*)a.Y)[tok * a.ldy + dst] = v;
          else ((_Float16*)a.Y)[tok * a.ldy + dst] = (_Float16)v;
        }
      }
    }
  };

  // the K steps of one row group: slot i holds step number i0 + i, and is refilled with the step a
  // whole ring later -- of this group, or of the next one when this group's (padded) steps run out
  auto k_loop = [&](int g) {
    for (int i0 = 0; i0 < nmine_p; i0 += kResRing) {
#pragma unroll
      for (int i = 0; i < kResRing; ++i) {
        if (i0 + i < nmine) compute(ring[i], wk + KW * (i0 + i));
        const bool wrap = i0 + i + kResRing >= nmine_p;
        load_a(ring[i], wrap ? g + 1 : g, wrap ? i0 + i + kResRing - nmine_p : i0 + i + kResRing);
      }
    }
  };
  if constexpr (ROWS) {
    // ---- row mode
    for (int g = 0; g < ngroups; ++g) {
      k_loop(g);
      const int64_t rb = rb_lo + (int64_t)g * RBW + wr;
      if (rb < rb_hi) store_rows(rb);
      zero_acc();
    }
    return;
  } else {
    // ---- K mode: one row group per workgroup
    k_loop(0);
    __syncthreads();                                        // every wave is done with the image
    float* red = (float*)smem;                              // [wave][token][65]
    {
      float* mine = red + (size_t)wave * kResTok * kResRedPitch;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int k = 0; k < 16; ++k)
            mine[(size_t)(j * 32 + tokl) * kResRedPitch + t * 32 + 8 * (k >> 2) + 4 * hB + (k & 3)] = acc[t][j][k];
    }
    __syncthreads();
    // element e of the group's output: (row block wr' = e / 4096, token, channel within the block)
    constexpr int NE = RBW * kResTok * 64;
    const int64_t zs = a.T * a.out;
    bool last = true;
    if (split) {
      float* mypart = a.part + (int64_t)blockIdx.z * zs;
      for (int e = tid; e < NE; e += 64 * kResWaves) {
        const int wrr = e >> 12, tok = (e >> 6) & 63, ch = e & 63;
        const int64_t o = (rb_lo + wrr) * 64 + ch, tk = t0 + tok;
        if (tk < a.T && o < a.out && rb_lo + wrr < rb_hi) {
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < KW; ++w) sum += red[((size_t)(w * RBW + wrr) * kResTok + tok) * kResRedPitch + ch];
          mypart[tk * a.out + o] = sum;
        }
      }
      // make the partial product visible to the whole device, then count this workgroup in
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __syncthreads();
      VNM_RS_LDS(unsigned) flag = (VNM_RS_LDS(unsigned))(smem + (size_t)kResWaves * kResTok * kResRedPitch * 4);
      if (tid == 0) *flag = arrive(a.arrivals + tile * a.R + rb_lo, a.tag);
      __syncthreads();
      last = *flag == gridDim.z;
      if (!last) return;
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    for (int e = tid; e < NE; e += 64 * kResWaves) {
      const int wrr = e >> 12, tok = (e >> 6) & 63, ch = e & 63;
      const int64_t o = (rb_lo + wrr) * 64 + ch, tk = t0 + tok;
      if (tk < a.T && o < a.out && rb_lo + wrr < rb_hi) {
        float sum = 0.f;
        if (split) {
          // all parts in ascending order, whoever arrived last: the sum is the same in every run
          for (unsigned z = 0; z < gridDim.z; ++z)
            sum += __builtin_nontemporal_load(a.part + (int64_t)z * zs + tk * a.out + o);
        } else {
#pragma unroll
          for (int w = 0; w < KW; ++w) sum += red[((size_t)(w * RBW + wrr) * kResTok + tok) * kResRedPitch + ch];
        }
        if (a.bias) sum += (float)a.bias[o];
        const int64_t dst = a.perm_out ? (int64_t)a.perm_out[o] : o;          // Eq. 6, P_o^T
        if (dst < 0 || dst >= a.out) continue;
        if (a.y_fp32) ((float*)a.Y)[tk * a.ldy + dst] = sum;
        else ((_Float16*)a.Y)[tk * a.ldy + dst] = (_Float16)sum;
      }
    }
  }
}

// ---- host side

static unsigned long long next_tag() {
  // 40-bit call tags: a process-wide counter started at a random value
  static std::atomic<unsigned long long> counter{[] {
    std::random_device rd;
    const unsigned long long t = (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
    return (((unsigned long long)rd() << 32) ^ rd() ^ t);
  }()};
  unsigned long long v;
  do { v = counter.fetch_add(1) & ((1ull << 40) - 1); } while (v == 0);
  return v;
}

int64_t resident_max_tokens_split() { return 256; }

struct ResPlan {
  bool ok = false, rows = false;
  int rbw = 8, pitch = 184, nsz = 0, parts = 1, rb_per = 8;
  int64_t tiles = 0, row_parts = 1;
  size_t lds = 0;
  unsigned ep_off = 0;
  int64_t part_bytes = 0, arrival_bytes = 0;
};

// How the resident kernel would run this product, if it can.  `scratch_bytes`: room for partial
// products and arrival slots (0 = none).
static ResPlan resident_plan(int64_t T, const Dims& d, int64_t scratch_bytes) {
  ResPlan p;
  if (!has_packed(d.V, d.M) || T <= 0) return p;
  const int64_t R = packed_row_blocks(d);
  p.tiles = (T + kResTok - 1) / kResTok;
  const int64_t rows_per_step = 8 * d.M;
  const size_t red_lds = (size_t)kResWaves * kResTok * kResRedPitch * 4 + 16;
  if (p.tiles > 0x7FFFFFFF) return p;
  if (T <= resident_max_tokens_split()) {
    // K mode.  Narrow image rows (less padding) keep the number of K parts down.
    p.pitch = 152;
    const int64_t nsz_max = (int64_t)(kResLdsMax / (size_t)(rows_per_step * p.pitch));
    if (nsz_max < 1) return p;
    int64_t parts = (d.S + nsz_max - 1) / nsz_max;
    // row blocks per workgroup: as many as still leave about one workgroup per CU
    int rbw = 1;
    for (int c : {8, 4, 2}) {
      if (p.tiles * ((R + c - 1) / c) * parts >= 240) { rbw = c; break; }
    }
    // few row blocks and few tokens: more K parts than LDS demands, while each keeps 8 steps or more
    while (p.tiles * ((R + rbw - 1) / rbw) * parts < 200 && d.S / (parts + 1) >= 8 && parts < 16) ++parts;
    if (parts > 16) return p;                               // more partial products than the scratch is sized for
    if (parts > 1) {
      p.part_bytes = (parts * T * d.out * 4 + 255) / 256 * 256;
      p.arrival_bytes = (p.tiles * R * 8 + 255) / 256 * 256;
      if (p.part_bytes + p.arrival_bytes > scratch_bytes) {
        // not enough scratch: fewer parts if LDS allows a single one, else not this kernel
        if ((d.S + nsz_max - 1) / nsz_max > 1) return p;
        parts = 1; p.part_bytes = p.arrival_bytes = 0;
      }
    }
    p.parts = (int)parts;
    p.nsz = (int)((d.S + parts - 1) / parts);
    p.parts = (int)((d.S + p.nsz - 1) / p.nsz);
    p.rbw = rbw; p.rb_per = rbw;
    p.row_parts = (R + rbw - 1) / rbw;
    const size_t img = (size_t)p.nsz * rows_per_step * p.pitch;
    p.lds = img > red_lds ? img : red_lds;
  } else {
    // row mode: the whole K range in LDS, next to the 8 epilogue strips; narrower rows if that is
    // what makes it fit
    const size_t strips = (size_t)kResWaves * kResEpBytes;
    const size_t room = 160 * 1024 - 64 - strips;
    p.pitch = 184;
    size_t img = (size_t)d.S * rows_per_step * p.pitch;
    if (img > room) { p.pitch = 152; img = (size_t)d.S * rows_per_step * p.pitch; }
    if (img > room) return p;
    p.nsz = (int)d.S; p.parts = 1; p.rbw = 8; p.rows = true;
    // Row parts: every workgroup loads its slice of X again, so few parts; but the grid should fill
    // the 256 CUs (one workgroup each).  Cost of a choice, in arbitrary units: rounds x (slice load +
    // groups per workgroup x (K steps + store)).
    const int64_t groups = (R + 7) / 8;
    double best = 1e300;
    int64_t best_rp = 1;
    for (int64_t rp = 1; rp <= groups; ++rp) {
      const int64_t gpw = (groups + rp - 1) / rp;
      const int64_t wgs = p.tiles * ((groups + gpw - 1) / gpw);
      const double rounds = (double)((wgs + 255) / 256);
      const double cost = rounds * ((double)img / 20e3 + (double)gpw * (0.3 * (double)d.S + 1.0));
      if (cost < best * 0.97) { best = cost; best_rp = rp; }
    }
    p.rb_per = (int)((groups + best_rp - 1) / best_rp) * 8;
    p.row_parts = (R + p.rb_per - 1) / p.rb_per;
    p.ep_off = (unsigned)((img + 15) / 16 * 16);
    p.lds = p.ep_off + strips;
  }
  if (p.row_parts > 65535 || p.parts > 65535) return p;
  p.ok = true;
  return p;
}

bool spmm_resident_applicable(int64_t T, const Dims& d, int64_t scratch_bytes) {
  return resident_plan(T, d, scratch_bytes).ok;
}

int64_t resident_scratch_bytes(int64_t T, const Dims& d) {
  // what the plan would use with unlimited scratch
  const ResPlan p = resident_plan(T, d, INT64_MAX / 2);
  return p.ok ? p.part_bytes + p.arrival_bytes : 0;
}

template <bool DUAL, int RBW, bool ROWS>
static int launch_res_cfg(const ResArgs& a, const ResPlan& p, hipStream_t st) {
  auto kern = spmm_resident_kernel<DUAL, RBW, ROWS>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(spmm_resident)")) return rc_lds;
  hipLaunchKernelGGL(kern, dim3((unsigned)p.tiles, (unsigned)p.row_parts, (unsigned)p.parts), dim3(64 * kResWaves),
                     p.lds + 16, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_resident_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

int launch_spmm_resident(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                         void* Y, int64_t ldy, int y_dtype, void* scratch, int64_t scratch_bytes,
                         const Fused& f, hipStream_t st) {
  const ResPlan p = resident_plan(T, d, scratch ? scratch_bytes : 0);
  if (!p.ok) return VNM_ERR_UNSUPPORTED;
  const PackedLayout pl = packed_layout(d);
  const char* pk = (const char*)packed;
  ResArgs a{};
  a.X = (const unsigned short*)X; a.T = T; a.ldx = ldx; a.in = d.in;
  a.pa = (const uint4*)(pk + pl.pa_off);
  a.pidx = (const unsigned*)(pk + pl.pidx_off);
  a.pcol = (const unsigned*)(pk + pl.pcol_off);
  a.out = d.out; a.R = packed_row_blocks(d); a.S = d.S; a.M = d.M; a.pitch = p.pitch;
  a.nsz = p.nsz; a.rb_per = p.rb_per;
  a.Y = Y; a.ldy = ldy; a.y_fp32 = y_dtype;
  a.vec_store = (ldy % 4 == 0) && (((uintptr_t)Y & (y_dtype == 0 ? 7 : 15)) == 0);
  a.bias = f.bias; a.perm_out = f.perm_out;
  a.ep_off = p.ep_off;
  a.wide_store = p.rows && y_dtype == 0 && !f.perm_out && ldy % 8 == 0 && (((uintptr_t)Y & 15) == 0);
  if (p.parts > 1) {
    a.part = (float*)scratch;
    a.arrivals = (unsigned long long*)((char*)scratch + p.part_bytes);
    a.tag = next_tag();
  }
  const bool dual = packed_tables(d.V) == 2;
  if (p.rows) return dual ? launch_res_cfg<true, 8, true>(a, p, st) : launch_res_cfg<false, 8, true>(a, p, st);
#define VNM_RES_GO(RBW)                                                                      \
  if (p.rbw == RBW) return dual ? launch_res_cfg<true, RBW, false>(a, p, st) : launch_res_cfg<false, RBW, false>(a, p, st);
  VNM_RES_GO(8) VNM_RES_GO(4) VNM_RES_GO(2) VNM_RES_GO(1)
#undef VNM_RES_GO
  return VNM_ERR_UNSUPPORTED;
}

}  // namespace vnm
