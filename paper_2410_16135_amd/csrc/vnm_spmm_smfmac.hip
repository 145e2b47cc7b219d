// vnm_spmm on the 2:4 sparse matrix cores of gfx950 (V_SMFMAC_F32_32X32X32_F16).
//
// Computes Y^T = W' . X^T so that the compressed weight is the sparse A operand (rows = output
// channels) and the activations are the dense B operand (columns = tokens).  What makes V:N:M differ
// from plain 2:4 (Appendix A) is that the B rows a row block needs are the 4 kept input columns of
// each of its column blocks, and they differ from row block to row block.  Design:
//
//   * A workgroup owns WR row blocks x (WT*TW) tokens.  Its raw X tile (all M columns of the current
//     K span) is staged once in LDS, TRANSPOSED to [input column][token], and shared by all WR row
//     blocks; the per-row-block gather happens when a wave reads its B operand: each
//     ds_read_b64_tr_b16 fetches, for 16 tokens, the 4 kept columns of one column block -- the rows
//     are chosen per lane from the packed column table -- and hands every lane the 4 K-consecutive
//     values of its token.  LDS read traffic is therefore exactly the gathered operand, with no
//     select arithmetic.
//   * The transposition is done in registers while staging: a thread loads a 4-token x 8-column
//     patch with four 16-byte global loads, interleaves halves with v_perm and writes eight 8-byte
//     LDS rows.
//   * A wave owns one row block (V rows = V/32 A tiles) x TW tokens (TW/32 B tiles); the A operand
//     (kept values in lane order + 2-bit positions) comes straight from the packed copy in global
//     memory with one 16-byte load per lane and tile; accumulators stay in registers for the whole
//     K loop.
#include "vnm_internal.h"

namespace vnm {

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
#define VNM_LDS(T) __attribute__((address_space(3))) T*

constexpr int kPitchPad = 64;  // bytes: successive staged rows start 16 banks apart

// 16 lanes x 8 bytes in, transposed out: lanes 4j..4j+3 of a 16-lane group address row j (16
// consecutive fp16 of it), and lane i receives element i of each of the 4 rows.
__device__ __forceinline__ h4 lds_read_tr(unsigned byte_addr) {
  const s4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((VNM_LDS(s4))(size_t)byte_addr);
  return __builtin_bit_cast(h4, v);
}

struct SpmmArgs {
  const _Float16* X; int64_t T, ldx;
  const uint4* pa; const unsigned short* pidx; const unsigned* pcol;
  int64_t out, in, R, S;
  int M, KS;
  void* Y; int64_t ldy;
  int vec_store;   // Y and ldy allow 4-wide stores
};

template <int V, int TW, int WR, int WT, typename OutT>
__global__ void __launch_bounds__(64 * WR * WT)
spmm_smfmac_kernel(const SpmmArgs a) {
  constexpr int AT = V / 32, BT = TW / 32, NT = 64 * WR * WT, TT = WT * TW;
  constexpr int P = TT * 2 + kPitchPad;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WT, wt = wave % WT;
  const int64_t r = (int64_t)blockIdx.y * WR + wr;
  const bool r_valid = r < a.R;
  const int64_t t0 = (int64_t)blockIdx.x * TT;
  const int M = a.M;

  f16v acc[AT][BT];
#pragma unroll
  for (int i = 0; i < AT; ++i)
#pragma unroll
    for (int j = 0; j < BT; ++j)
#pragma unroll
      for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.f;

  // B-operand lane roles
  const int hB = lane >> 5, tg = (lane >> 4) & 1, kq = (lane & 15) >> 2, q = lane & 3;
  const unsigned lds0 = (unsigned)(size_t)(VNM_LDS(unsigned char))smem;
  const unsigned tokoff = (unsigned)((wt * TW + tg * 16 + q * 4) * 2);

  constexpr int NPT = TT / 4;  // 4-token patches along the token axis
  for (int64_t s0 = 0; s0 < a.S; s0 += a.KS) {
    const int nks = (int)((a.S - s0) < a.KS ? (a.S - s0) : a.KS);
    // ---- stage the raw X tile, transposed
    const int npc = nks * M;                                       // 8-column patches
    const int64_t col0 = s0 * 8 * M;
    for (int item = tid; item < npc * NPT; item += NT) {
      const int pt = item % NPT, pc = item / NPT;
      const int64_t col = col0 + pc * 8;
      const int64_t tok = t0 + 4 * pt;
      uint4 g[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        g[j] = make_uint4(0, 0, 0, 0);
        if (col < a.in && tok + j < a.T) g[j] = *(const uint4*)(a.X + (tok + j) * a.ldx + col);
      }
      unsigned char* dst = smem + (size_t)(pc * 8) * P + pt * 8;
      const unsigned d[4][4] = {{g[0].x, g[1].x, g[2].x, g[3].x}, {g[0].y, g[1].y, g[2].y, g[3].y},
                                {g[0].z, g[1].z, g[2].z, g[3].z}, {g[0].w, g[1].w, g[2].w, g[3].w}};
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        uint2 lo, hi;
        lo.x = __builtin_amdgcn_perm(d[p][1], d[p][0], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(d[p][3], d[p][2], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(d[p][1], d[p][0], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(d[p][3], d[p][2], 0x07060302u);
        *(uint2*)(dst + (size_t)(2 * p) * P) = lo;
        *(uint2*)(dst + (size_t)(2 * p + 1) * P) = hi;
      }
    }
    __syncthreads();
    // ---- multiply
    if (r_valid) {
      for (int ks = 0; ks < nks; ++ks) {
        const int64_t rs = r * a.S + s0 + ks;
        h8 av[AT];
#pragma unroll
        for (int i = 0; i < AT; ++i) {
          const uint4 w = a.pa[(rs * AT + i) * 64 + lane];
          av[i] = __builtin_bit_cast(h8, w);
        }
        unsigned idxw[(AT + 1) / 2];
        if (AT == 1) idxw[0] = a.pidx[rs * 64 + lane];
        else {
#pragma unroll
          for (int i = 0; i < AT / 2; ++i) idxw[i] = ((const unsigned*)a.pidx)[(rs * 64 + lane) * (AT / 2) + i];
        }
        const unsigned pc4 = a.pcol[rs * 8 + hB * 4 + kq];
        unsigned addr[4];
#pragma unroll
        for (int m = 0; m < 4; ++m)
          addr[m] = lds0 + (unsigned)(ks * 8 * M + ((pc4 >> (8 * m)) & 255u)) * P + tokoff;
#pragma unroll
        for (int j = 0; j < BT; ++j) {
          const h4 b0 = lds_read_tr(addr[0] + j * 64);
          const h4 b1 = lds_read_tr(addr[1] + j * 64);
          const h4 b2 = lds_read_tr(addr[2] + j * 64);
          const h4 b3 = lds_read_tr(addr[3] + j * 64);
          h16 bv;
#pragma unroll
          for (int e = 0; e < 4; ++e) { bv[e] = b0[e]; bv[4 + e] = b1[e]; bv[8 + e] = b2[e]; bv[12 + e] = b3[e]; }
#pragma unroll
          for (int i = 0; i < AT; ++i) {
            if (i & 1)
              acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(av[i], bv, acc[i][j], (int)idxw[i / 2], 0, 1);
            else
              acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(av[i], bv, acc[i][j], (int)idxw[i / 2], 0, 0);
          }
        }
      }
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds, per (A tile, B tile, jq), 4 consecutive output channels of one token
  if (!r_valid) return;
  OutT* Y = (OutT*)a.Y;
  const int tokl = lane & 31;
#pragma unroll
  for (int j = 0; j < BT; ++j) {
    const int64_t tok = t0 + wt * TW + j * 32 + tokl;
    if (tok >= a.T) continue;
#pragma unroll
    for (int i = 0; i < AT; ++i) {
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const int64_t o = r * V + i * 32 + 8 * jq + 4 * hB;
        OutT* dst = Y + tok * a.ldy + o;
        const float v0 = acc[i][j][4 * jq], v1 = acc[i][j][4 * jq + 1], v2 = acc[i][j][4 * jq + 2],
                    v3 = acc[i][j][4 * jq + 3];
        if (a.vec_store && o + 3 < a.out) {
          if (sizeof(OutT) == 2) {
            h4 pk = {(_Float16)v0, (_Float16)v1, (_Float16)v2, (_Float16)v3};
            *(h4*)dst = pk;
          } else {
            f4 pk = {v0, v1, v2, v3};
            *(f4*)dst = pk;
          }
        } else {
          if (o < a.out) dst[0] = (OutT)v0;
          if (o + 1 < a.out) dst[1] = (OutT)v1;
          if (o + 2 < a.out) dst[2] = (OutT)v2;
          if (o + 3 < a.out) dst[3] = (OutT)v3;
        }
      }
    }
  }
}

bool spmm_smfmac_applicable(const void* X, int64_t ldx, const Dims& d) {
  return has_packed(d.V, d.M) && d.in % 8 == 0 && ldx % 8 == 0 && ((uintptr_t)X & 15) == 0;
}

template <int V, int TW, int WR, int WT, typename OutT>
static int launch_cfg(const SpmmArgs& a, hipStream_t st) {
  constexpr int TT = WT * TW;
  constexpr int P = TT * 2 + kPitchPad;
  const size_t lds = (size_t)a.KS * 8 * a.M * P;
  auto kern = spmm_smfmac_kernel<V, TW, WR, WT, OutT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute(spmm_smfmac)"); return VNM_ERR_HIP; }
    attr_set = true;
  }
  dim3 grid((unsigned)((a.T + TT - 1) / TT), (unsigned)((a.R + WR - 1) / WR));
  hipLaunchKernelGGL(kern, grid, dim3(64 * WR * WT), lds, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "spmm_smfmac_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

int launch_spmm_smfmac(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                       void* Y, int64_t ldy, int y_dtype, hipStream_t st) {
  const PackedLayout pl = packed_layout(d);
  const char* p = (const char*)packed;
  SpmmArgs a;
  a.X = (const _Float16*)X; a.T = T; a.ldx = ldx;
  a.pa = (const uint4*)(p + pl.pa_off);
  a.pidx = (const unsigned short*)(p + pl.pidx_off);
  a.pcol = (const unsigned*)(p + pl.pcol_off);
  a.out = d.out; a.in = d.in; a.R = d.R; a.S = d.S; a.M = d.M;
  a.KS = 128 / (8 * d.M) > 0 ? 128 / (8 * d.M) : 1;
  a.Y = Y; a.ldy = ldy;
  a.vec_store = (ldy % 4 == 0) && (((uintptr_t)Y & (y_dtype == 0 ? 7 : 15)) == 0);
  if (T > (int64_t)65535 * 128) return VNM_ERR_UNSUPPORTED;
#define VNM_GO(Vv, TWv, WRv, WTv)                                                       \
  return y_dtype == 0 ? launch_cfg<Vv, TWv, WRv, WTv, _Float16>(a, st)                 \
                      : launch_cfg<Vv, TWv, WRv, WTv, float>(a, st)
  switch (d.V) {
    case 32: VNM_GO(32, 256, 4, 1);
    case 64: VNM_GO(64, 128, 4, 1);
    case 128: VNM_GO(128, 64, 4, 1);
  }
#undef VNM_GO
  return VNM_ERR_UNSUPPORTED;
}

}  // namespace vnm
