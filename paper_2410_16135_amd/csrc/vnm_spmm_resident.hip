// vnm_spmm without a staging pass, for the layers of the DeiT-shaped configurations (Section 5.1),
// where a separate staging pass costs as much as the product: a short K range (qkv, proj, fc1), or
// a long one with few output channels (fc2).
//
// A workgroup owns 64 tokens.  It reads its slice of X straight from the caller's matrix and turns
// it around on the way into LDS: [raw input column][token], the order the transposing LDS read of
// the matrix-core kernel wants (vnm_spmm_smfmac.hip: one ds_read_b64_tr_b16 fetches, for 16 tokens,
// the 4 kept columns of a column block, the rows chosen per lane from the packed column table).
// Each of the 8 waves works on 64-row blocks of its own and streams their weight operands through a
// ring of registers, requested ahead of the one it multiplies.  Two shapes:
//   * whole K in LDS: the image is built once, after one barrier nothing is written to it any more,
//     and the waves take the row blocks of the workgroup's range in turn (any number of them);
//   * K in chunks: the accumulators of all the workgroup's row blocks stay in registers (at most 2
//     per wave, i.e. 1024 output channels) while X streams through two image buffers, one barrier
//     per chunk; the next chunk travels in registers while the current one is multiplied.
// fp16 results are turned around in a private strip of LDS per wave and leave as whole 128-byte
// runs of Y rows.
//
// Tried and dropped: the same kernel for 33..256 tokens at any K, with K cut into parts over
// workgroups and waves and the fp32 partial products summed by the workgroup that arrives last at
// a tile.  Every workgroup then re-reads and re-transposes its slice of X, and about 60 GB/s into
// one CU make that, and the last workgroup's reading of all parts, slower than the staging pass +
// streaming kernel + reduction kernel it was meant to replace (Llama-shaped layers at 64:2:5, per
// call: q 22-37 us against 19-28, gate 50-104 against 24-40).
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
constexpr int kResEpPitch = 144;       // fp16 epilogue: bytes per token row of a wave's strip
constexpr int kResEpBytes = 32 * kResEpPitch;

// pieces of X per thread and chunk the chunked form is built for (a chunk is one ring of K steps:
// 6, or 4 with two held row blocks per wave; M <= 8)
constexpr int resident_chunk_pieces(int rpw) { return rpw == 2 ? 4 : 6; }

struct ResArgs {
  const unsigned short* X; int64_t T, ldx, in;
  const uint4* pa; const unsigned* pidx; const unsigned* pcol;
  int64_t out, R, S;                   // R: 64-row blocks of the packed copy
  int M, pitch;                        // pitch: bytes between image rows in LDS (a multiple of 8)
  int csz, nchunks;                    // K steps per chunk (S when nchunks == 1), number of chunks
  unsigned buf_bytes;                  // one image buffer (there are two when nchunks > 1)
  int rb_per;                          // row blocks per workgroup
  void* Y; int64_t ldy; int y_fp32, vec_store;
  int wide_store;                      // fp16 Y with 16-byte stores through the LDS strips at ep_off
  unsigned ep_off;
  const _Float16* bias; const int* perm_out;
};

// DUAL: the 64-row block carries one column table per 32-row tile (V = 32 patterns).
// CHUNKED: K streams through two image buffers instead of lying in LDS as a whole.
// RPW: row blocks whose accumulators a wave holds at a time (2 only with K in chunks).
template <bool DUAL, int RPW, bool CHUNKED>
__global__ void __launch_bounds__(64 * kResWaves) spmm_resident_kernel(const ResArgs a) {
  static_assert(CHUNKED || RPW == 1, "two held row blocks only with K in chunks");
  constexpr int NT = DUAL ? 2 : 1;
  constexpr int RING = RPW == 2 ? 4 : 6;                    // A operands a wave keeps in flight
  // 16-byte pieces of X a thread holds at a time: a whole chunk (it travels in registers while the
  // previous one is multiplied), or a batch of the one-off image
  constexpr int NX = CHUNKED ? resident_chunk_pieces(RPW) : 14;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int M = a.M, P = a.pitch;
  const int64_t tile = blockIdx.x, t0 = tile * kResTok;
  const int nchunks = CHUNKED ? a.nchunks : 1, csz = a.csz;
  const int csz_p = (csz + RING - 1) / RING * RING;         // a segment's steps, padded to whole rings

  // ---- roles
  const int hB = lane >> 5, tg = (lane >> 4) & 1, kq = (lane & 15) >> 2, q = lane & 3;
  const unsigned tokoff = (unsigned)((tg * 16 + q * 4) * 2);
  const int64_t rb_lo = (int64_t)blockIdx.y * a.rb_per;
  const int64_t rb_hi = rb_lo + a.rb_per < a.R ? rb_lo + a.rb_per : a.R;
  constexpr int kBatch = kResWaves * RPW;                   // row blocks the workgroup holds at a time
  const int nbatch = (int)((rb_hi - rb_lo + kBatch - 1) / kBatch);

  // A wave's work is a list of segments -- batch by batch, chunk by chunk, held row block by held
  // row block -- of csz K steps each, padded to a multiple of the ring size so that step i of a
  // segment always sits in ring slot i % RING (slots are registers, their index must be a
  // constant).  Padding steps are loaded like real ones (from a valid address) and never multiplied.
  struct AOp { uint4 w[2]; unsigned idx; unsigned pc[NT]; };
  // Operands are requested in exactly the order the steps are multiplied in, RING steps ahead, by a
  // cursor of scalars: (batch, chunk, held row block, step) and, per segment, the number of the
  // segment's first (row block, K step) pair in the packed copy and of the row block's last one.  A
  // step costs an add and a minimum; the multiplications happen once per segment.  Every load is
  // unconditional, pairs beyond the ends are clamped to valid ones.  32-bit byte offsets: the plan
  // admits at most 2^21 (row block, K step) pairs of 2 KiB.
  int l_bt = 0, l_c = 0, l_r = 0, l_step = 0;
  unsigned l_base = 0, l_lim = 0;
  auto seg_setup = [&]() {
    int64_t rb = rb_lo + (int64_t)l_bt * kBatch + l_r * kResWaves + wave;
    rb = rb < a.R ? rb : a.R - 1;
    l_base = (unsigned)(rb * a.S + (int64_t)l_c * csz);
    l_lim = (unsigned)(rb * a.S + a.S - 1);
  };
  seg_setup();
  const unsigned lane_a = (unsigned)lane * 16u, lane_i = (unsigned)lane * 4u;
  const unsigned lane_c = (unsigned)((hB * 4 + kq) * NT) * 4u;
  auto load_next = [&](AOp& o) {
    unsigned rs = l_base + (unsigned)l_step;
    rs = rs < l_lim ? rs : l_lim;
    const char* pw = (const char*)a.pa + (rs * 2048u + lane_a);
    o.w[0] = *(const uint4*)pw;
    o.w[1] = *(const uint4*)(pw + 1024);
    o.idx = *(const unsigned*)((const char*)a.pidx + (rs * 256u + lane_i));
#pragma unroll
    for (int t = 0; t < NT; ++t) o.pc[t] = *(const unsigned*)((const char*)a.pcol + (rs * (unsigned)(32 * NT) + lane_c + 4u * t));
    if (++l_step == csz_p) {
      l_step = 0;
      if (++l_r == RPW) {
        l_r = 0;
        if (++l_c == nchunks) { l_c = 0; ++l_bt; }
      }
      seg_setup();
    }
  };
  AOp ring[RING];

  // ---- X -> LDS, transposed.  Eight lanes share a token (a whole 128-byte line of its row per
  // load), a wave-wide load covers 8 tokens x 8 chunks of 16 bytes; every lane then stores its 8
  // columns to 8 image rows, two bytes each.  Rows beyond T and columns beyond `in` become zero (the
  // packed copy holds zero weights there, and zero times whatever else LDS held could be NaN).
  const int tsub = lane >> 3, csub = lane & 7;
  // pieces [first, first + NX) of this thread for chunk c: piece n is unit wave + 8 n, unit u =
  // (chunk group u >> 3, token group u & 7) -- so all pieces of a thread belong to one token, number
  // wave * 8 + tsub of the tile, and piece n starts (first + n) * 64 + csub * 8 columns into the
  // chunk's span.  The loads are unconditional (the compiler then knows how many are in flight and
  // can let the weight operands requested after them stay in flight while X is parked) and cheap to address: one row pointer per thread (a
  // valid row also for tokens beyond T), a 32-bit column clamped to the last 8 that exist in the span
  // and in the row; what a clamped piece brings is dropped when it is parked.
  const int x_tok = wave * 8 + tsub;
  const unsigned short* x_row = a.X + (t0 + x_tok < a.T ? (t0 + x_tok) * a.ldx : 0);
  auto x_load = [&](uint4 (&xw)[NX], int c, int first) {
    const int64_t col0 = (int64_t)c * csz * 8 * M;
    const int64_t sleft = a.S - (int64_t)c * csz;
    const int CH = (int)(sleft < csz ? sleft : csz) * M;    // 16-byte chunks per token
    const int64_t span_end = col0 + (int64_t)CH * 8;
    const unsigned col_last = (unsigned)((span_end < a.in ? span_end : a.in) - 8);
    const unsigned col_first = (unsigned)col0 + (unsigned)(csub * 8);
#pragma unroll
    for (int n = 0; n < NX; ++n) {
      const unsigned col = col_first + (unsigned)((first + n) * 64);
      xw[n] = *(const uint4*)(x_row + (col < col_last ? col : col_last));
    }
    // the loads that follow in the program (weight operands) must follow in the instruction stream
    // too -- loads return in order, and X is what is waited for first
    __builtin_amdgcn_sched_barrier(0);
  };
  auto x_park = [&](const uint4 (&xw)[NX], int c, int first, unsigned buf) {
    const int64_t col0 = (int64_t)c * csz * 8 * M;
    const int64_t sleft = a.S - (int64_t)c * csz;
    const int CH = (int)(sleft < csz ? sleft : csz) * M;
    const int CHz = csz * M;                                // a short last chunk is padded with zero rows
#pragma unroll
    for (int n = 0; n < NX; ++n) {
      const int tok = x_tok, ch = (first + n) * 8 + csub;
      if (ch < CHz) {
        const bool ok = ch < CH && t0 + tok < a.T && col0 + ch * 8 < a.in;
        const uint4 v = ok ? xw[n] : make_uint4(0, 0, 0, 0);
        unsigned char* d = smem + buf + (size_t)(ch * 8) * P + tok * 2;
        const unsigned w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          *(unsigned short*)(d + (size_t)(2 * e) * P) = (unsigned short)(w4[e] & 0xFFFFu);
          *(unsigned short*)(d + (size_t)(2 * e + 1) * P) = (unsigned short)(w4[e] >> 16);
        }
      }
    }
  };
  // Loads return in order: the first pieces of X are requested first, then the first ring of weight
  // operands (from HBM; their latency runs under the work on X), then X is parked.
  uint4 xn[CHUNKED ? NX : 1];                               // the chunk that travels (chunked form only)
  const int nimg = CHUNKED ? nbatch * nchunks : 1;          // images this workgroup builds
  if constexpr (CHUNKED) {
    x_load(xn, 0, 0);
#pragma unroll
    for (int i = 0; i < RING; ++i) load_next(ring[i]);
    x_park(xn, 0, 0, 0);
    if (nimg > 1) x_load(xn, nchunks > 1 ? 1 : 0, 0);       // under the first chunk's multiplications
  } else {
    const int npieces = (csz * M + 7) / 8;                  // per thread: chunk groups of 8 x 8 token groups over 8 waves
    uint4 xw[NX];
    x_load(xw, 0, 0);
#pragma unroll
    for (int i = 0; i < RING; ++i) load_next(ring[i]);
    x_park(xw, 0, 0, 0);
    for (int first = NX; first < npieces; first += NX) {
      x_load(xw, 0, first);
      x_park(xw, 0, first, 0);
    }
  }
  __syncthreads();

  rs_f16 acc[RPW][2][2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int k = 0; k < 16; ++k) acc[r][t][j][k] = 0.f;
  };

  const unsigned lds0 = (unsigned)(size_t)(VNM_RS_LDS(unsigned char))smem;
  // one K step: ls = step within the image at byte offset buf; per token half, four transposing reads
  // at the rows the packed table names, and their matrix instructions
  auto compute = [&](rs_f16 (&ac)[2][2], const AOp& o, unsigned buf, int ls) {
    const int ix = (int)o.idx;
    const unsigned base = lds0 + buf + (unsigned)(ls * 8 * M) * (unsigned)P + tokoff;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      unsigned row[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) row[m] = base + __umul24((o.pc[t] >> (8 * m)) & 255u, (unsigned)P);
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
          ac[0][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(rs_h8, o.w[0]), bv, ac[0][j], ix, 0, 0);
        if (!DUAL || t == 1)
          ac[1][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(rs_h8, o.w[1]), bv, ac[1][j], ix, 0, 1);
      }
    }
  };

  const int tokl = lane & 31;
  // Accumulator element 4 jq + e of tile (t, j) is channel rb * 64 + t * 32 + 8 jq + 4 hB + e of token
  // t0 + 32 j + tokl.
  auto store_rows = [&](const rs_f16 (&acc)[2][2], int64_t rb) {
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
          // Y is written once and not read again here: a non-temporal store keeps it from displacing
          // X and the weight operands in the caches
          if (tok < a.T) {
            typedef unsigned rs_u4 __attribute__((ext_vector_type(4)));
            const rs_u4 vv = {v.x, v.y, v.z, v.w};
            __builtin_nontemporal_store(vv, (rs_u4*)(Yh + tok * a.ldy + rb * 64 + c8 * 8));
          }
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
                __builtin_nontemporal_store(pk, (rs_f4*)((float*)a.Y + tok * a.ldy + o));
              } else {
                rs_h4 pk = {(_Float16)(acc[t][j][4 * jq] + bv[0]), (_Float16)(acc[t][j][4 * jq + 1] + bv[1]),
                            (_Float16)(acc[t][j][4 * jq + 2] + bv[2]), (_Float16)(acc[t][j][4 * jq + 3] + bv[3])};
                __builtin_nontemporal_store(pk, (rs_h4*)((_Float16*)a.Y + tok * a.ldy + o));
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

  // ---- the loops
  // (Reading the next step's B operands from LDS ahead of the current step's matrix instructions, with
  // a second set of operand registers, measured no faster: 81.9 against 80.7 us over a DeiT-small
  // block.  What a step used to wait for was the scalar unit, shared by the CU's 8 waves: the address
  // arithmetic of the operand loads, about 45 scalar instructions per wave and step before the
  // cursor above, took more of it than the four matrix instructions take of a SIMD.)
  int img = 0;                                              // image being multiplied
  for (int bt = 0; bt < nbatch; ++bt) {
    zero_acc();
    for (int c = 0; c < nchunks; ++c) {
      const unsigned buf = CHUNKED ? (unsigned)(img & 1) * a.buf_bytes : 0u;
      const int64_t sleft = a.S - (int64_t)c * csz;
      const int nsc = (int)(sleft < csz ? sleft : csz);     // real steps of this chunk
#pragma unroll
      for (int r = 0; r < RPW; ++r) {
        const int64_t rb = rb_lo + (int64_t)bt * kBatch + r * kResWaves + wave;
        const bool mine = rb < rb_hi;
        for (int i0 = 0; i0 < csz_p; i0 += RING) {
#pragma unroll
          for (int i = 0; i < RING; ++i) {
            if (i0 + i < nsc && mine) compute(acc[r], ring[i], buf, i0 + i);
            load_next(ring[i]);
          }
        }
      }
      if constexpr (CHUNKED) {
        // the next image goes into the other buffer (whose last readers passed the previous
        // barrier), the one after it starts travelling
        const int c1 = c + 1 == nchunks ? 0 : c + 1, c2 = c1 + 1 == nchunks ? 0 : c1 + 1;   // chunks of the next two images
        if (img + 1 < nimg) x_park(xn, c1, 0, (unsigned)((img + 1) & 1) * a.buf_bytes);
        if (img + 2 < nimg) x_load(xn, c2, 0);
        __syncthreads();
        ++img;
      }
    }
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
      const int64_t rb = rb_lo + (int64_t)bt * kBatch + r * kResWaves + wave;
      if (rb < rb_hi) store_rows(acc[r], rb);
    }
  }
}

// ---- host side

struct ResPlan {
  bool ok = false;
  int pitch = 184, csz = 0, nchunks = 1, rpw = 1, rb_per = 8;
  int64_t tiles = 0, row_parts = 1;
  unsigned buf_bytes = 0, ep_off = 0;
  size_t lds = 0;
};

// How the resident kernel would run this product, if it can.
static ResPlan resident_plan(int64_t T, const Dims& d) {
  ResPlan p;
  if (!has_packed(d.V, d.M) || T <= 0) return p;
  const int64_t R = packed_row_blocks(d);
  p.tiles = (T + kResTok - 1) / kResTok;
  if (p.tiles > 0x7FFFFFFF || R * d.S > ((int64_t)1 << 21)) return p;    // the kernel addresses the packed copy with 32-bit offsets
  const int64_t rows_per_step = 8 * d.M;
  const size_t strips = (size_t)kResWaves * kResEpBytes;
  const size_t room = 160 * 1024 - 64 - strips;             // LDS left for images next to the epilogue strips
  const int64_t groups = (R + 7) / 8;
  // whole K in LDS; narrower image rows if that is what makes it fit
  p.pitch = 184;
  size_t img = (size_t)d.S * rows_per_step * p.pitch;
  if (img > room) { p.pitch = 152; img = (size_t)d.S * rows_per_step * p.pitch; }
  if (img <= room) {
    p.csz = (int)d.S; p.nchunks = 1; p.rpw = 1;
    // Row parts: every workgroup builds the image again, so few parts; but the grid should fill the
    // 256 CUs (one workgroup each).  Cost of a choice, arbitrary units: rounds x (image + groups per
    // workgroup x (K steps + store)).
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
    p.buf_bytes = (unsigned)((img + 15) / 16 * 16);
    p.ep_off = p.buf_bytes;
    p.lds = p.ep_off + strips;
    p.ok = p.row_parts <= 65535;
    return p;
  }
  // K in chunks of one ring of steps, two image buffers; all row blocks of the layer in one
  // workgroup's registers (8 waves x at most 2), enough token tiles to occupy the chip, and the
  // pieces of a chunk must fit the registers that carry it (kResNX per thread)
  p.rpw = R <= kResWaves ? 1 : 2;
  p.csz = p.rpw == 2 ? 4 : 6;
  p.pitch = 152;
  if (R > 2 * kResWaves || p.tiles < 128 || (p.csz * d.M + 7) / 8 > resident_chunk_pieces(p.rpw)) return p;
  p.nchunks = (int)((d.S + p.csz - 1) / p.csz);
  p.buf_bytes = (unsigned)(((size_t)p.csz * rows_per_step * p.pitch + 15) / 16 * 16);
  if (2 * (size_t)p.buf_bytes > room) return p;
  p.rb_per = (int)R; p.row_parts = 1;
  p.ep_off = 2 * p.buf_bytes;
  p.lds = p.ep_off + strips;
  p.ok = true;
  return p;
}

bool spmm_resident_applicable(int64_t T, const Dims& d) { return resident_plan(T, d).ok; }

template <bool DUAL, int RPW, bool CHUNKED>
static int launch_res_cfg(const ResArgs& a, const ResPlan& p, hipStream_t st) {
  auto kern = spmm_resident_kernel<DUAL, RPW, CHUNKED>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(spmm_resident)")) return rc_lds;
  hipLaunchKernelGGL(kern, dim3((unsigned)p.tiles, (unsigned)p.row_parts), dim3(64 * kResWaves), p.lds + 16, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_resident_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

int launch_spmm_resident(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                         void* Y, int64_t ldy, int y_dtype, const Fused& f, hipStream_t st) {
  const ResPlan p = resident_plan(T, d);
  if (!p.ok) return VNM_ERR_UNSUPPORTED;
  const PackedLayout pl = packed_layout(d);
  const char* pk = (const char*)packed;
  ResArgs a{};
  a.X = (const unsigned short*)X; a.T = T; a.ldx = ldx; a.in = d.in;
  a.pa = (const uint4*)(pk + pl.pa_off);
  a.pidx = (const unsigned*)(pk + pl.pidx_off);
  a.pcol = (const unsigned*)(pk + pl.pcol_off);
  a.out = d.out; a.R = packed_row_blocks(d); a.S = d.S; a.M = d.M; a.pitch = p.pitch;
  a.csz = p.csz; a.nchunks = p.nchunks; a.buf_bytes = p.buf_bytes; a.rb_per = p.rb_per;
  a.Y = Y; a.ldy = ldy; a.y_fp32 = y_dtype;
  a.vec_store = (ldy % 4 == 0) && (((uintptr_t)Y & (y_dtype == 0 ? 7 : 15)) == 0);
  a.bias = f.bias; a.perm_out = f.perm_out;
  a.ep_off = p.ep_off;
  a.wide_store = y_dtype == 0 && !f.perm_out && ldy % 8 == 0 && (((uintptr_t)Y & 15) == 0);
  const bool dual = packed_tables(d.V) == 2;
  if (p.nchunks == 1) return dual ? launch_res_cfg<true, 1, false>(a, p, st) : launch_res_cfg<false, 1, false>(a, p, st);
  if (p.rpw == 2) return dual ? launch_res_cfg<true, 2, true>(a, p, st) : launch_res_cfg<false, 2, true>(a, p, st);
  return dual ? launch_res_cfg<true, 1, true>(a, p, st) : launch_res_cfg<false, 1, true>(a, p, st);
}

}  // namespace vnm
