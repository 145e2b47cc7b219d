// vnm_spmm for few tokens (decode, small batches): no staging pass; at most 32 tokens always (a workspace
// is optional then: split K for few row blocks), up to 256 tokens where the resident-X kernel further down
// can take them in groups (skinny_plan).
//
// With so few tokens the product is a stream of the compressed weight through the matrix cores at
// HBM rate; what matters is that every byte of it is requested early and read once.  One workgroup
// owns one 64-row block of the packed copy and the whole K range; its 8 waves take the
// K steps round-robin, each into private accumulators, and add them up through LDS at the end, so
// no partial products leave the chip.  K is walked in phases of P steps: the A operands and the
// slice of X of phase p+1 are requested before phase p is multiplied and are parked (X: in a
// second LDS buffer) after it.  X stays token-major in LDS, [token][raw column] with an odd
// number of dwords per row; a lane assembles its B operand -- for its token, the 4 kept columns
// of 4 column blocks -- with 16 two-byte LDS reads at the offsets of the packed column table
// (conflict-free: lanes differ in the row).  That is 16 LDS instructions per matrix instruction
// pair, far below what the streaming rate needs; the transposing staged layout of the many-token
// kernel would cost a second launch.  For at most 16 tokens a second kernel (further down) keeps the
// whole slice of X in LDS and runs 16 waves with a short ring of weight operands each instead.
//
// Measured and dropped: dealing the (row block, K step) pairs out evenly to one workgroup per compute
// unit and adding the parts up inside the kernel (parts to memory with device-scope stores, one arrival
// counter per row block, the last workgroup to arrive sums in a fixed order).  It was exact and used all
// 256 units, but the L2 slices of different XCDs do not snoop each other, so parts and counters travel
// through memory: store acknowledged, counter returned, parts read back are three dependent round
// trips of about 2 us each.  16 tokens, 64:2:5, back to back: 4096 x 4096 18.0 us against 11.0 us for
// one workgroup per row block; 11008 x 4096 21.6 against 12.9; 4096 x 11008 18.3 against 14.4 for
// split K plus the reduction launch.  A kernel boundary is the cheaper device-wide hand-over here.
//
// Also measured and dropped, for up to 16 tokens: the slice of X transposed into LDS ([raw column][16
// tokens], 32 bytes per column, one row left empty after every 8) and the B operand fetched with four
// transposing reads per step as in the many-token kernels, instead of 16 two-byte reads.  The steps got
// shorter (3.8 -> 3.2 us for the 13 steps of a wave; what they wait for is mostly the second round of
// weight loads, not their own instructions), but parking X took longer than it saved (3.8 -> 5.9 us
// with two-byte stores, more with pairs of lanes exchanging halves to store dwords): 12.6 against
// 11.6 us on 4096 x 4096, 14.1 against 13.0 us on 11008 x 4096.  A ring of 13 operands (every weight
// of a wave requested before X is complete) made it worse still: the weights crowd out the loads of X
// that the barrier waits for.
//
// Also measured and dropped, on the 16-wave form of that kernel: the B operand of a step gathered once per
// wave instead of once per lane (lane (token, K group) reads 8 halfwords of X and stores them as 16 bytes
// of a wave-private strip [token][32 compacted K]; every lane reads its operand back with two 16-byte
// reads: 11 LDS instructions and a dozen integer instructions per lane and step instead of 16 and about
// 50).  Same results, slower: the store and the read-back are two more dependent LDS round trips per step
// (device time per call at 16 tokens, weights from HBM: 4096 x 4096 10.8 against 9.6 us, 11008 x 4096 13.3
// against 13.0; at 32 tokens 18.6 against 18.3 us on 11008 x 4096).
#include "vnm_internal.h"

namespace vnm {

typedef _Float16 sk_h8 __attribute__((ext_vector_type(8)));
typedef _Float16 sk_h16 __attribute__((ext_vector_type(16)));
typedef float sk_f16 __attribute__((ext_vector_type(16)));
typedef unsigned sk_u8 __attribute__((ext_vector_type(8)));

constexpr int kSkWaves = 8;      // waves per workgroup
constexpr int kSkSPW = 4;        // K steps per wave and phase, at most
constexpr int kSkNX = 8;         // 16-byte pieces of X per thread and phase, at most
constexpr int kSkHalfTileMaxWorkgroups = 256;   // the device's compute units

struct SkinnyArgs {
  const unsigned short* X; int64_t T, ldx, in;
  const uint4* pa; const unsigned short* pidx; const uint4* pcol;
  int64_t out, S;
  int M, P;                      // P: K steps per phase, a multiple of 8, at most 32
  void* Y; int64_t ldy; int y_fp32;
  // split K: workgroup (r, z) walks phases [z * npz, min(nph, (z + 1) * npz)) and writes its fp32
  // partial product at Y + z * z_stride elements (a scratch then; summed by splitk_reduce)
  int npz; int64_t z_stride;
  int nsz;                       // resident-X kernel: K steps per workgroup (split K as above, counted in steps)
  int tgroups;                   // resident-X kernel: groups of 16 tokens, one workgroup each per (row block, K piece)
  int64_t R;                     // resident-X kernel: 64-row blocks of the packed copy
  // fused epilogue (null = none): bias per weight row, destination channel per weight row
  const _Float16* bias; const int* perm_out;
};

// DUAL: the 64-row block carries one column table per 32-row tile (V = 32 patterns) instead of one
// for both; TT: token rows held in LDS (16 or 32)
template <bool DUAL, int TT>
__global__ void __launch_bounds__(64 * kSkWaves) spmm_skinny_kernel(const SkinnyArgs a) {
  constexpr int AT = 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t r = blockIdx.x;
  const int M = a.M, P = a.P;
  const int64_t S = a.S;
  const int ncolP = P * 8 * M;                       // raw columns of a phase
  const int pitch = ncolP * 2 + 4;                   // bytes per token row: odd number of dwords
  const int bufB = (TT * pitch + 15) & ~15;
  const int nph_all = (int)((S + P - 1) / P);
  const int p_begin = (int)blockIdx.y * a.npz;
  const int p_end = p_begin + a.npz < nph_all ? p_begin + a.npz : nph_all;
  const int spw = P / kSkWaves;
  // X pieces of this thread: piece i is (token, chunk) number tid + 512 i in row-major order
  const int CH = P * M;
  const int tok_first = tid / CH, ch_first = tid - tok_first * CH;
  const int dtok = 512 / CH, dch = 512 - dtok * CH;

  // All global loads below are unconditional (out-of-range pieces read a valid dummy address and
  // are zeroed or ignored later): loads under a branch would make the number of outstanding loads
  // unknown to the compiler, which then drains every one of them before the first use of any.
  uint4 xw[kSkNX];
  auto x_valid = [&](int tok, int ch, int64_t col0) { return tok < TT && tok < a.T && col0 + ch * 8 < a.in; };
  auto load_x = [&](int p) {
    const int64_t col0 = (int64_t)p * ncolP;
    int tok = tok_first, ch = ch_first;
#pragma unroll
    for (int i = 0; i < kSkNX; ++i) {
      const unsigned short* src = x_valid(tok, ch, col0) ? a.X + tok * a.ldx + col0 + ch * 8 : a.X;
      xw[i] = *(const uint4*)src;
      ch += dch; tok += dtok;
      if (ch >= CH) { ch -= CH; ++tok; }
    }
  };
  auto store_x = [&](int buf, int p) {
    const int64_t col0 = (int64_t)p * ncolP;
    int tok = tok_first, ch = ch_first;
#pragma unroll
    for (int i = 0; i < kSkNX; ++i) {
      if (tok < TT) {
        const uint4 v = x_valid(tok, ch, col0) ? xw[i] : make_uint4(0, 0, 0, 0);
        unsigned* d = (unsigned*)(smem + (size_t)buf * bufB + (size_t)tok * pitch + ch * 16);
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
      }
      ch += dch; tok += dtok;
      if (ch >= CH) { ch -= CH; ++tok; }
    }
  };

  struct AOp { uint4 w[AT]; unsigned idx; uint4 pc, pc2; };
  const int hB = lane >> 5;
  auto load_a = [&](AOp (&o)[kSkSPW], int p) {
#pragma unroll
    for (int i = 0; i < kSkSPW; ++i) {
      // steps beyond the phase or beyond S re-read the last valid one; compute() skips them
      int64_t s = (int64_t)p * P + wave + kSkWaves * (i < spw ? i : spw - 1);
      s = s < S ? s : S - 1;
      const int64_t rs = r * S + s;
#pragma unroll
      for (int t = 0; t < AT; ++t) o[i].w[t] = a.pa[(rs * AT + t) * 64 + lane];
      o[i].idx = ((const unsigned*)a.pidx)[rs * 64 + lane];
      if (DUAL) { o[i].pc = a.pcol[rs * 4 + hB * 2]; o[i].pc2 = a.pcol[rs * 4 + hB * 2 + 1]; }
      else o[i].pc = a.pcol[rs * 2 + hB];
    }
  };

  sk_f16 acc[AT];
#pragma unroll
  for (int t = 0; t < AT; ++t)
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[t][k] = 0.f;

  const int tokl = (TT == 32) ? (lane & 31) : (lane & 15);      // TT = 16: lanes 16..31 repeat 0..15
  auto compute = [&](const AOp (&o)[kSkSPW], int buf, int p) {
#pragma unroll
    for (int i = 0; i < kSkSPW; ++i) {
      const int64_t s = (int64_t)p * P + wave + kSkWaves * i;
      if (i < spw && s < S) {
        const unsigned char* row = smem + (size_t)buf * bufB + (size_t)tokl * pitch + (size_t)(wave + kSkWaves * i) * 16 * M;
        // column tables as [kq] -> 4 packed row offsets (byte m = load m); DUAL interleaves the
        // two tables: (kq 0 table 0, kq 0 table 1, kq 1 table 0, ...)
        unsigned pc[2][4];
        if (DUAL) {
          pc[0][0] = o[i].pc.x; pc[1][0] = o[i].pc.y; pc[0][1] = o[i].pc.z; pc[1][1] = o[i].pc.w;
          pc[0][2] = o[i].pc2.x; pc[1][2] = o[i].pc2.y; pc[0][3] = o[i].pc2.z; pc[1][3] = o[i].pc2.w;
        } else {
          pc[0][0] = o[i].pc.x; pc[0][1] = o[i].pc.y; pc[0][2] = o[i].pc.z; pc[0][3] = o[i].pc.w;
        }
        const int ix = (int)o[i].idx;
#pragma unroll
        for (int t = 0; t < (DUAL ? 2 : 1); ++t) {
          sk_u8 bw;
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            // element 4m + kq of the B operand: kept column kq of column block blk(m, h)
            unsigned v[4];
#pragma unroll
            for (int kq = 0; kq < 4; ++kq) v[kq] = *(const unsigned short*)(row + 2 * ((pc[t][kq] >> (8 * m)) & 255u));
            bw[2 * m] = v[0] | (v[1] << 16);
            bw[2 * m + 1] = v[2] | (v[3] << 16);
          }
          const sk_h16 bv = __builtin_bit_cast(sk_h16, bw);
          if (!DUAL || t == 0)
            acc[0] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(sk_h8, o[i].w[0]), bv, acc[0], ix, 0, 0);
          if (!DUAL || t == 1)
            acc[1] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(sk_h8, o[i].w[1]), bv, acc[1], ix, 0, 1);
        }
      }
    }
  };

  AOp cur[kSkSPW], nxt[kSkSPW];
  load_x(p_begin);
  load_a(cur, p_begin);
  store_x(p_begin & 1, p_begin);
  __syncthreads();
  for (int p = p_begin; p < p_end; ++p) {
    const bool more = p + 1 < p_end;
    const int pn = more ? p + 1 : p;            // the last phase re-requests itself (unused)
    load_x(pn);
    load_a(nxt, pn);
    compute(cur, p & 1, p);
    if (more) store_x((p + 1) & 1, pn);
#pragma unroll
    for (int i = 0; i < kSkSPW; ++i) cur[i] = nxt[i];
    __syncthreads();
  }

  // sum of the 8 waves' accumulators through LDS, [wave][token][rows + 1] fp32, then the store.
  // Accumulator element j of lane l is row 8 (j / 4) + 4 (l / 32) + j % 4 of the tile, token l % 32.
  constexpr int RW = AT * 32;
  float* red = (float*)smem;
  if ((lane & 31) < TT) {
    float* mine = red + ((size_t)wave * TT + (lane & 31)) * (RW + 1);
#pragma unroll
    for (int t = 0; t < AT; ++t)
#pragma unroll
      for (int j = 0; j < 16; ++j) mine[t * 32 + 8 * (j >> 2) + 4 * hB + (j & 3)] = acc[t][j];
  }
  __syncthreads();
  for (int e = tid; e < TT * RW; e += 64 * kSkWaves) {
    const int tok = e / RW, rw = e - tok * RW;
    const int64_t o = r * RW + rw;
    if (tok < a.T && o < a.out) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < kSkWaves; ++w) sum += red[((size_t)w * TT + tok) * (RW + 1) + rw];
      if (a.bias) sum += (float)a.bias[o];
      const int64_t dst = a.perm_out ? (int64_t)a.perm_out[o] : o;          // Eq. 6, P_o^T
      if (dst < 0 || dst >= a.out) continue;
      if (a.y_fp32) ((float*)a.Y)[(int64_t)blockIdx.y * a.z_stride + tok * a.ldy + dst] = sum;
      else ((_Float16*)a.Y)[tok * a.ldy + dst] = (_Float16)sum;
    }
  }
}

// Up to 16 tokens whose slice of X fits LDS as a whole (16 rows of the workgroup's K range: in <= ~4800
// columns unsplit, more with split K): X is fetched once, up front, and then nothing is written to LDS
// any more, so the K loop needs no barrier and no registers for X.  A workgroup has 16 waves; every wave
// takes the steps wave, wave + 16, ... and keeps a short ring of A operands requested ahead of the one it
// multiplies.  All loads are unconditional (clamped to the last step), so the compiler can wait for
// exactly the operand it uses next.  What keeps the weight stream going is the number of waves on the
// compute unit, not the depth of a wave's ring: device time per call at 16 tokens, 64:2:5, weights from
// HBM, on 4096 x 4096 / 11008 x 4096 / 4096 x 11008 --
//   8 waves, ring 8:  12.2 / 14.7 / 17.2 us      8 waves, ring 4:  10.9 / 13.2 / 14.4 us
//   16 waves, ring 4: 10.6 / 13.7 / 14.7 us      16 waves, ring 3: 10.1 / 13.4 / 14.9 us
//   16 waves, ring 2:  9.6 / 13.0 / 14.2 us      16 waves, ring 1:  9.5 / 12.5 / 14.2 us
// (rings of 10 and 13 had measured no better than 8 before).  Every further operand in flight is another
// load instruction queued in the unit's memory pipeline in front of the ones some wave is waiting for.
constexpr int kSkWavesR = 16;    // waves per workgroup of the resident-X kernel
constexpr int kSkNXR = 10;       // 16-byte pieces of X per thread, at most (16 rows of at most 9216 bytes)

// HALF: one workgroup per 32-row tile (blockIdx.z picks the tile of the 64-row block) instead of one per
// block -- twice the workgroups where a matrix has too few row blocks to occupy the compute units; each
// fetches the whole slice of X but only its tile's weights.
template <bool DUAL, bool HALF, int RB, int TT>
__global__ void __launch_bounds__(64 * kSkWavesR) spmm_skinny_resident_kernel(const SkinnyArgs a) {
  constexpr int AT = 2;
  constexpr int NT = HALF ? 1 : AT;                  // tiles of this workgroup
  const int t0 = HALF ? (int)blockIdx.z : 0;         // its first tile
  // operands requested ahead per wave (see the table above)
  constexpr int kSkRing = 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // RB row blocks per workgroup, kSkWavesR / RB waves each; a row block beyond the last one (odd count) is
  // computed as a copy of the last and not stored
  constexpr int WPB = kSkWavesR / RB;
  const int rbi = wave / WPB, wsub = wave % WPB;
  const int64_t r_own = (int64_t)blockIdx.x * RB + rbi;
  const int64_t r = r_own < a.R ? r_own : a.R - 1;
  const int M = a.M;
  const int64_t S = a.S;
  // blockIdx.y = K piece * token groups + token group; a group is TT token rows of X and Y
  const int tg = (int)(blockIdx.y % (unsigned)a.tgroups);
  const int64_t ky = blockIdx.y / (unsigned)a.tgroups;
  const int64_t Tg = a.T - TT * tg < TT ? a.T - TT * tg : TT;       // tokens of this group (at least one)
  const unsigned short* Xg = a.X + (int64_t)tg * TT * a.ldx;
  const int64_t s_lo = ky * a.nsz;
  const int64_t s_hi = s_lo + a.nsz < S ? s_lo + a.nsz : S;
  const int ncol = a.nsz * 8 * M;                    // raw columns of a workgroup's K range
  const int pitch = ncol * 2 + 4;                    // bytes per token row: odd number of dwords
  const int64_t col0 = s_lo * 8 * M;

  struct AOp { uint4 w[NT]; unsigned idx; uint4 pc, pc2; };
  const int hB = lane >> 5;
  auto load_a = [&](AOp& o, int64_t s) {
    s = s < S ? s : S - 1;                           // beyond the range: a valid operand that is never used
    const int64_t rs = r * S + s;
#pragma unroll
    for (int t = 0; t < NT; ++t) o.w[t] = a.pa[(rs * AT + t0 + t) * 64 + lane];
    o.idx = ((const unsigned*)a.pidx)[rs * 64 + lane];
    if (DUAL) { o.pc = a.pcol[rs * 4 + hB * 2]; o.pc2 = a.pcol[rs * 4 + hB * 2 + 1]; }
    else o.pc = a.pcol[rs * 2 + hB];
  };
  AOp ring[kSkRing];

  // X slice -> LDS, [token][raw column], in 16-byte pieces.  One wave-wide load takes a block of 4 token
  // rows x 16 chunks (256-byte runs of a row: whole cache lines; in LDS the four rows start an odd number
  // of dwords apart, so the 64 lanes' stores fall into 64 different banks); block number b = wave + 16 i is
  // (group of 4 token rows b % (TT / 4), chunk group b / (TT / 4)).  Rows beyond T and columns beyond `in` become zero.  The
  // first ring of weight operands is requested right after X: loads return in order, so X (from L2) is
  // not held up behind the weights (from HBM), and the weights travel while X is being parked in LDS.
  {
    const int CH = ncol / 8;
    const int c_lo = lane & 15, rsub = lane >> 4;
    constexpr int NB = DUAL ? 2 : 1;                 // one batch where the registers allow it
    constexpr int HB = kSkNXR / NB;
    // All blocks of a thread lie in one token row (16 is a multiple of TT / 4), CG * 128 columns apart:
    // one row pointer (a valid row also for tokens beyond T) and a 32-bit column, clamped to the last
    // 8 columns that exist in the K range and in the row -- what a clamped load brings is dropped below.
    constexpr int NG = TT / 4;                       // groups of 4 token rows
    const int x_tok = (wave % NG) * 4 + rsub;
    const unsigned short* x_row = Xg + (x_tok < Tg ? x_tok * a.ldx : 0);
    const int64_t span_end = col0 + ncol;
    const unsigned col_last = (unsigned)((span_end < a.in ? span_end : a.in) - 8);
    const unsigned col_first = (unsigned)col0 + (unsigned)(((wave / NG) * 16 + c_lo) * 8);
    constexpr int CG = kSkWavesR / NG;              // chunk groups of 16 pieces taken per round of wave-wide loads
#pragma unroll
    for (int half = 0; half < NB; ++half) {
      uint4 xw[HB];
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        const unsigned col = col_first + (unsigned)((half * HB + i) * (CG * 128));
        xw[i] = *(const uint4*)(x_row + (col < col_last ? col : col_last));
      }
      // keep the compiler from moving the weight loads below in front of these: loads return in order
      __builtin_amdgcn_sched_barrier(0);
      if (half == 0) {
#pragma unroll
        for (int i = 0; i < kSkRing; ++i) load_a(ring[i], s_lo + wsub + WPB * i);
      }
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        const int tok = x_tok, ch = ((wave / NG) + CG * (half * HB + i)) * 16 + c_lo;
        if (ch < CH) {
          const bool ok = tok < Tg && col0 + ch * 8 < a.in;
          const uint4 v = ok ? xw[i] : make_uint4(0, 0, 0, 0);
          unsigned* d = (unsigned*)(smem + (size_t)tok * pitch + ch * 16);
          d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
      }
    }
  }
  __syncthreads();

  sk_f16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[t][k] = 0.f;

  const int tokl = lane & (TT - 1);                  // TT = 16: lanes 16..31 repeat tokens 0..15
  auto compute = [&](const AOp& o, int64_t s) {
    const unsigned char* row = smem + (size_t)tokl * pitch + (size_t)(s - s_lo) * 16 * M;
    unsigned pc[2][4];
    if (DUAL) {
      pc[0][0] = o.pc.x; pc[1][0] = o.pc.y; pc[0][1] = o.pc.z; pc[1][1] = o.pc.w;
      pc[0][2] = o.pc2.x; pc[1][2] = o.pc2.y; pc[0][3] = o.pc2.z; pc[1][3] = o.pc2.w;
    } else {
      pc[0][0] = o.pc.x; pc[0][1] = o.pc.y; pc[0][2] = o.pc.z; pc[0][3] = o.pc.w;
    }
    const int ix = (int)o.idx;
    if (HALF) {
      // the one tile of this workgroup: its column table (DUAL) or the shared one, its half of the index word
      const int tb = DUAL ? t0 : 0;
      sk_u8 bw;
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        unsigned v[4];
#pragma unroll
        for (int kq = 0; kq < 4; ++kq) v[kq] = *(const unsigned short*)(row + 2 * (((tb ? pc[1][kq] : pc[0][kq]) >> (8 * m)) & 255u));
        bw[2 * m] = v[0] | (v[1] << 16);
        bw[2 * m + 1] = v[2] | (v[3] << 16);
      }
      const sk_h16 bv = __builtin_bit_cast(sk_h16, bw);
      if (t0 == 0) acc[0] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(sk_h8, o.w[0]), bv, acc[0], ix, 0, 0);
      else acc[0] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(sk_h8, o.w[0]), bv, acc[0], ix, 0, 1);
      return;
    }
#pragma unroll
    for (int t = 0; t < (DUAL ? 2 : 1); ++t) {
      sk_u8 bw;
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        unsigned v[4];
#pragma unroll
        for (int kq = 0; kq < 4; ++kq) v[kq] = *(const unsigned short*)(row + 2 * ((pc[t][kq] >> (8 * m)) & 255u));
        bw[2 * m] = v[0] | (v[1] << 16);
        bw[2 * m + 1] = v[2] | (v[3] << 16);
      }
      const sk_h16 bv = __builtin_bit_cast(sk_h16, bw);
      if (!DUAL || t == 0)
        acc[0] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(sk_h8, o.w[0]), bv, acc[0], ix, 0, 0);
      if (!DUAL || t == 1)
        acc[NT - 1] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(sk_h8, o.w[NT - 1]), bv, acc[NT - 1], ix, 0, 1);
    }
  };

  for (int64_t sb = s_lo + wsub; sb < s_hi; sb += WPB * kSkRing) {
#pragma unroll
    for (int i = 0; i < kSkRing; ++i) {
      const int64_t s = sb + WPB * i;
      if (s < s_hi) compute(ring[i], s);
      load_a(ring[i], s + WPB * kSkRing);
    }
  }
  __syncthreads();                                   // every wave is done with X: the reduction reuses its LDS

  constexpr int RW = AT * 32;                        // rows of a block
  constexpr int RT = NT * 32;                        // rows of this workgroup
  float* red = (float*)smem;
  if ((lane & 31) < TT) {
    float* mine = red + ((size_t)wave * TT + (lane & 31)) * (RW + 1);
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < 16; ++j) mine[t * 32 + 8 * (j >> 2) + 4 * hB + (j & 3)] = acc[t][j];
  }
  __syncthreads();
  for (int e = tid; e < RB * TT * RT; e += 64 * kSkWavesR) {
    const int rb = e / (TT * RT), e1 = e - rb * (TT * RT);
    const int tok = e1 / RT, rw = e1 - tok * RT;
    const int64_t o = ((int64_t)blockIdx.x * RB + rb) * RW + t0 * 32 + rw;
    if (tok < Tg && o < a.out) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < WPB; ++w) sum += red[((size_t)(rb * WPB + w) * TT + tok) * (RW + 1) + rw];
      if (a.bias) sum += (float)a.bias[o];
      const int64_t dst = a.perm_out ? (int64_t)a.perm_out[o] : o;          // Eq. 6, P_o^T
      if (dst < 0 || dst >= a.out) continue;
      const int64_t yrow = TT * tg + tok;
      if (a.y_fp32) ((float*)a.Y)[ky * a.z_stride + yrow * a.ldy + dst] = sum;
      else ((_Float16*)a.Y)[yrow * a.ldy + dst] = (_Float16)sum;
    }
  }
}

// LDS of the resident-X kernel for nsz K steps and tt token rows per workgroup; 0 if they do not fit
static size_t skinny_resident_lds(int M, int64_t nsz, int tt) {
  const size_t x = (size_t)tt * ((size_t)nsz * 16 * M + 4);
  const size_t red = (size_t)kSkWavesR * tt * (2 * 32 + 1) * 4;
  const size_t lds = x > red ? x : red;
  // kSkNXR wave-wide loads per wave cover the slice: tt / 4 groups of token rows x ceil(nsz M / 16) chunk groups
  if (lds > 150 * 1024 || (size_t)(tt / 4) * (((size_t)nsz * M + 15) / 16) > (size_t)kSkWavesR * kSkNXR) return 0;
  return lds;
}

template <bool DUAL, bool HALF, int RB, int TT>
static int launch_skinny_resident(const SkinnyArgs& a, int64_t R, int KS, size_t lds, hipStream_t st) {
  auto kern = spmm_skinny_resident_kernel<DUAL, HALF, RB, TT>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(spmm_skinny_resident)")) return rc_lds;
  hipLaunchKernelGGL(kern, dim3((unsigned)((R + RB - 1) / RB), (unsigned)(KS * a.tgroups), HALF ? 2u : 1u),
                     dim3(64 * kSkWavesR), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_skinny_resident_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

// How the resident-X kernel serves T tokens, if it can.
//   tt      token rows per workgroup: 16, or 32 where groups of 16 would not fit (a group of 32 costs a
//           workgroup the same instructions per K step and twice the slice of X)
//   rb      row blocks per workgroup (the waves are dealt out to them; one slice of X for all)
//   ks      workgroups along K (> 1: fp32 partial products in the scratch, summed by splitk_reduce)
// All (row, K, token-group) workgroups must fit the compute units at once: one whose turn comes later
// starts from nothing when the first ones end.  Candidates: 16 tokens and one or two row blocks per
// workgroup; 32 tokens and one, two or four row blocks with K split as far as the slice of X needs.
struct SkPlan { int tt, rb, groups; int64_t ks, nsz; size_t lds; bool half; };

static bool skinny_plan(int64_t T, const Dims& d, bool have_scratch, int64_t scratch_bytes, SkPlan* p) {
  const int64_t R = packed_row_blocks(d);
  // candidates (tokens per workgroup, smallest and largest number of row blocks per workgroup), in the order
  // they are tried.  Up to 32 tokens one group of 32 comes before two groups of 16 with two row blocks each
  // (11008 x 4096 at 32 tokens: 16.9 against 18.5 us); beyond, the groups of 16 come first (4096 x 4096 at 128
  // tokens: 15.4 us against 16.6 us for groups of 32 with K in two pieces).
  const int cand[4][3] = {{16, 1, 1}, {T <= 32 ? 32 : 16, T <= 32 ? 1 : 2, T <= 32 ? 4 : 2}, {16, 2, 2}, {32, 1, 4}};
  for (int ci = 0; ci < (T > 16 ? 4 : 1); ++ci) {
    const int tt = cand[ci][0];
    const int groups = (int)((T + tt - 1) / tt);
    if (tt == 16 && groups == 1 && cand[ci][1] > 1) continue;
    for (int rb = cand[ci][1]; rb <= cand[ci][2]; rb *= 2) {
      const int64_t Re = (R + rb - 1) / rb;                               // workgroups along the rows
      if (T > 16 && Re * groups > kSkHalfTileMaxWorkgroups) continue;
      int64_t ks = 1;
      if (tt == 16) {
        // K is split (while the workgroups still fit the 256 CUs at once) only beyond 128 K steps, into
        // pieces of at least 32: a shorter K is done sooner by one workgroup per row block than by
        // several plus the reduction launch (measured at 64:2:5 and 64:2:8 on 4096 x 4096: 12.6 / 10.7 us
        // unsplit against 13.5 / 12.7 us split in four; 4096 x 11008: 15.2 us split in four against
        // 18.1 us split in two)
        if (have_scratch && T <= skinny_max_tokens() && Re * groups <= 128 && d.S > 128) {
          ks = 256 / (Re * groups);
          if (ks > 16) ks = 16;
          if (ks > d.S / 32) ks = d.S / 32;
        }
        // a slice of X that does not fit LDS (wide blocks, M = 16: 16 tokens x 32 M bytes per K step):
        // more pieces, down to 16 K steps each, while the workgroups still fit the compute units
        if (have_scratch && T <= skinny_max_tokens())
          while (ks < 16 && (d.S + ks - 1) / ks >= 16 && !skinny_resident_lds(d.M, (d.S + ks - 1) / ks, tt) &&
                 Re * groups * (ks + 1) <= kSkHalfTileMaxWorkgroups) ++ks;
      } else {
        // 32 tokens per workgroup: as few pieces of K as the slice of X allows
        while (ks <= 8 && (d.S + ks - 1) / ks >= 32 && !skinny_resident_lds(d.M, (d.S + ks - 1) / ks, tt)) ++ks;
        if (ks > 1 && !have_scratch) continue;
        if (Re * groups * ks > kSkHalfTileMaxWorkgroups) continue;
      }
      while (ks > 1 && ks * T * d.out * 4 > scratch_bytes) --ks;
      const int64_t nsz = (d.S + ks - 1) / ks;
      // below 32 steps per workgroup (16 where K had to be split for LDS) there is nothing to keep in flight
      const size_t lds = nsz >= (ks > 1 ? 16 : 32) ? skinny_resident_lds(d.M, nsz, tt) : 0;
      if (!lds) continue;
      const int64_t KSr = (d.S + nsz - 1) / nsz;
      p->tt = tt; p->rb = rb; p->groups = groups; p->ks = KSr; p->nsz = nsz; p->lds = lds;
      // one workgroup per 32-row tile while even those leave compute units idle
      p->half = tt == 16 && rb == 1 && 2 * R * KSr * groups <= kSkHalfTileMaxWorkgroups;
      return true;
    }
  }
  return false;
}

int64_t skinny_max_tokens() { return 32; }

template <bool DUAL, int TT>
static int launch_skinny_cfg(const SkinnyArgs& a, int64_t R, int KS, hipStream_t st) {
  const size_t bufB = ((size_t)TT * (a.P * 16 * a.M + 4) + 15) & ~(size_t)15;
  size_t lds = 2 * bufB;
  const size_t red = (size_t)kSkWaves * TT * (2 * 32 + 1) * 4;
  if (red > lds) lds = red;
  auto kern = spmm_skinny_kernel<DUAL, TT>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(spmm_skinny)")) return rc_lds;
  hipLaunchKernelGGL(kern, dim3((unsigned)R, (unsigned)KS), dim3(64 * kSkWaves), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_skinny_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

// 33 to 256 tokens where the resident-X kernel can take them in groups (see skinny_plan); scratch_bytes:
// what the caller can offer for split-K partial products
bool skinny_groups_applicable(int64_t T, const Dims& d, int64_t scratch_bytes) {
  if (T <= skinny_max_tokens() || T > 256 || !has_packed(d.V, d.M)) return false;
  SkPlan p;
  return skinny_plan(T, d, scratch_bytes > 0, scratch_bytes, &p);
}

int launch_spmm_skinny(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                       void* Y, int64_t ldy, int y_dtype, void* scratch, int64_t scratch_bytes,
                       const Fused& f, hipStream_t st) {
  // one to four tokens: the vector-ALU stream of vnm_spmm_gemv.hip
  if (spmm_gemv_applicable(T, ldx, d)) return launch_spmm_gemv(X, T, ldx, packed, d, Y, ldy, y_dtype, f, st);
  const PackedLayout pl = packed_layout(d);
  const char* p = (const char*)packed;
  const bool dual = packed_tables(d.V) == 2;
  const int64_t R = packed_row_blocks(d);
  if (R > 0x7FFFFFFF) return VNM_ERR_UNSUPPORTED;
  SkinnyArgs a{};
  a.X = (const unsigned short*)X; a.T = T; a.ldx = ldx; a.in = d.in;
  a.pa = (const uint4*)(p + pl.pa_off);
  a.pidx = (const unsigned short*)(p + pl.pidx_off);
  a.pcol = (const uint4*)(p + pl.pcol_off);
  a.out = d.out; a.S = d.S; a.M = d.M;
  a.Y = Y; a.ldy = ldy; a.y_fp32 = y_dtype;
  a.bias = f.bias; a.perm_out = f.perm_out;
  const int TT = T <= 16 ? 16 : 32;
  // the resident-X kernel where it applies (T <= 16, or more tokens in groups of 16 or 32 per workgroup:
  // the packed weight is then requested once per group and comes from HBM once; device time per call at
  // 64:2:5 on 4096 x 4096 at 32 tokens: 9.7 us against 14.6 us for the phased kernel)
  SkPlan pl2;
  if (skinny_plan(T, d, scratch != nullptr, scratch_bytes, &pl2)) {
    a.nsz = (int)pl2.nsz; a.z_stride = 0; a.tgroups = pl2.groups; a.R = R;
    const int KSr = (int)pl2.ks;
    if (KSr > 1) {
      a.Y = scratch; a.ldy = d.out; a.y_fp32 = 1; a.z_stride = T * d.out;
      a.bias = nullptr; a.perm_out = nullptr;                             // applied by the reduction
    }
    int rc = VNM_ERR_UNSUPPORTED;
#define VNM_SK_LAUNCH(H, RBV, TTV) \
    rc = dual ? launch_skinny_resident<true, H, RBV, TTV>(a, R, KSr, pl2.lds, st) : launch_skinny_resident<false, H, RBV, TTV>(a, R, KSr, pl2.lds, st)
    if (pl2.tt == 16) {
      if (pl2.rb == 2) VNM_SK_LAUNCH(false, 2, 16);
      else if (pl2.half) VNM_SK_LAUNCH(true, 1, 16);
      else VNM_SK_LAUNCH(false, 1, 16);
    } else {
      if (pl2.rb == 4) VNM_SK_LAUNCH(false, 4, 32);
      else if (pl2.rb == 2) VNM_SK_LAUNCH(false, 2, 32);
      else VNM_SK_LAUNCH(false, 1, 32);
    }
#undef VNM_SK_LAUNCH
    if (rc != VNM_OK || KSr == 1) return rc;
    return launch_splitk_reduce(scratch, KSr, T, d.out, Y, ldy, y_dtype, f, st);
  }
  if (T > skinny_max_tokens()) return VNM_ERR_UNSUPPORTED;               // the phased kernel holds at most 32 token rows
  // steps per phase: a multiple of the 8 waves, at most 32, with at most kSkNX pieces of X per thread
  // (TT * P * M <= 512 * kSkNX), which also keeps the two LDS buffers below 132 KiB
  int P = 512 * kSkNX / (TT * d.M) / 8 * 8;
  P = P > 32 ? 32 : (P < 8 ? 8 : P);
  a.P = P;
  // A workgroup's phases run one memory round trip after the other, so a long K on few row blocks
  // is latency-bound.  With scratch, and while all workgroups still fit the 256 CUs at once (a second
  // round costs more than it saves), K is split over several workgroups per row block; their fp32
  // partial products are summed by a second kernel.
  const int nph = (int)((d.S + P - 1) / P);
  int KS = 1;
  a.npz = nph; a.z_stride = 0;
  if (scratch && nph > 1 && R <= 128) {
    int64_t ks = 256 / R;
    if (ks > 16) ks = 16;
    if (ks > nph) ks = nph;
    while (ks > 1 && ks * T * d.out * 4 > scratch_bytes) --ks;
    if (ks > 1) {
      a.npz = (int)((nph + ks - 1) / ks);
      KS = (nph + a.npz - 1) / a.npz;
    }
  }
  if (KS > 1) {
    a.Y = scratch; a.ldy = d.out; a.y_fp32 = 1; a.z_stride = T * d.out;
    a.bias = nullptr; a.perm_out = nullptr;                               // applied by the reduction
  }
  int rc = VNM_ERR_UNSUPPORTED;
  if (!dual) rc = TT == 16 ? launch_skinny_cfg<false, 16>(a, R, KS, st) : launch_skinny_cfg<false, 32>(a, R, KS, st);
  else rc = TT == 16 ? launch_skinny_cfg<true, 16>(a, R, KS, st) : launch_skinny_cfg<true, 32>(a, R, KS, st);
  if (rc != VNM_OK || KS == 1) return rc;
  return launch_splitk_reduce(scratch, KS, T, d.out, Y, ldy, y_dtype, f, st);
}

}  // namespace vnm
