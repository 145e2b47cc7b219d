// vnm_decompress, vnm_pack and the generic (scalar) vnm_spmm kernel.
#include "vnm_internal.h"

namespace vnm {

// ---------------------------------------------------------------- decompress (Appendix A, inverse)
// One thread per element of W' [out x in]: look up the block's kept columns and the row's two
// positions, emit the kept value (bit copy) or +0.0.  Stores are fully coalesced.
__global__ void __launch_bounds__(256)
decompress_kernel(const unsigned short* __restrict__ values, const unsigned char* __restrict__ meta,
                  const unsigned char* __restrict__ colidx, int64_t out, int64_t in, int V, int M,
                  int64_t B, unsigned short* __restrict__ Wd, int64_t ldw, int64_t row0) {
  const int64_t col = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = row0 + blockIdx.y;
  if (col >= in) return;
  const int64_t b = col / M;
  const int ci = (int)(col - b * M);
  const int64_t r = row / V;
  const uchar4 k4 = *(const uchar4*)(colidx + (r * B + b) * 4);
  const unsigned char k[4] = {k4.x, k4.y, k4.z, k4.w};
  const unsigned byte = meta[row * ((B + 1) / 2) + (b >> 1)];
  const unsigned nib = (b & 1) ? (byte >> 4) : (byte & 15u);
  const unsigned pair = *(const unsigned*)(values + row * 2 * B + 2 * b);
  unsigned short w = 0;
  if (k[nib & 3] == ci) w = (unsigned short)(pair & 0xFFFFu);
  else if (k[nib >> 2] == ci) w = (unsigned short)(pair >> 16);
  Wd[row * ldw + col] = w;
}

int launch_decompress(const void* values, const void* meta, const void* colidx, const Dims& d,
                      void* W_out, int64_t ldw, hipStream_t st) {
  for (int64_t r0 = 0; r0 < d.out; r0 += 65535) {                // grid.y limit
    const int64_t rows = d.out - r0 < 65535 ? d.out - r0 : 65535;
    dim3 grid((unsigned)((d.in + 255) / 256), (unsigned)rows);
    hipLaunchKernelGGL(decompress_kernel, grid, dim3(256), 0, st, (const unsigned short*)values,
                       (const unsigned char*)meta, (const unsigned char*)colidx, d.out, d.in, d.V,
                       d.M, d.B, (unsigned short*)W_out, ldw, r0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e, "decompress_kernel"); return VNM_ERR_HIP; }
  }
  return VNM_OK;
}

// ---------------------------------------------------------------- pack
// Re-orders the canonical triple into the operand order of V_SMFMAC_F32_32X32X32_F16.
// A K step covers 8 column blocks (32 compacted K).  In a 32-row tile, lane l = i + 32*h holds the
// row i, and its 8 values e = 0..7 are the two kept values of blocks 4h + e/2 of the step; the 2-bit
// position of value e sits at bits [2e+1 : 2e] of the lane's 16-bit index word.  Blocks beyond the
// last real one get value 0 and positions (0, 1).
__global__ void __launch_bounds__(256)
pack_kernel(const unsigned short* __restrict__ values, const unsigned char* __restrict__ meta,
            const unsigned char* __restrict__ colidx, int V, int M, int64_t R, int64_t Rp, int64_t B, int64_t S,
            unsigned short* __restrict__ pa, unsigned short* __restrict__ pidx,
            unsigned char* __restrict__ pcol) {
  // Rp packed row blocks of 64 rows (2 tiles of 32); R row blocks of V rows in the pattern
  const int NT = V == 32 ? 2 : 1;                 // column tables per packed row block
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = Rp * S * 2 * 64;
  if (gid < total) {
    const int lane = (int)(gid & 63);
    int64_t rest = gid >> 6;
    const int at = (int)(rest & 1); rest >>= 1;
    const int64_t s = rest % S;
    const int64_t rp = rest / S;
    const int i = lane & 31, h = lane >> 5;
    const int64_t row = rp * 64 + at * 32 + i;
    const bool row_ok = row < R * V;              // rows beyond the padded matrix: value 0, positions (0, 1)
    unsigned short v[8];
    unsigned idx = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int64_t b = s * 8 + 4 * h + g;
      unsigned pair = 0, nib = 4;                                  // (0, 1)
      if (b < B && row_ok) {
        pair = *(const unsigned*)(values + row * 2 * B + 2 * b);
        const unsigned byte = meta[row * ((B + 1) / 2) + (b >> 1)];
        nib = (b & 1) ? (byte >> 4) : (byte & 15u);
      }
      v[2 * g] = (unsigned short)(pair & 0xFFFFu);
      v[2 * g + 1] = (unsigned short)(pair >> 16);
      idx |= nib << (4 * g);
    }
    uint4 q;
    q.x = v[0] | ((unsigned)v[1] << 16); q.y = v[2] | ((unsigned)v[3] << 16);
    q.z = v[4] | ((unsigned)v[5] << 16); q.w = v[6] | ((unsigned)v[7] << 16);
    *(uint4*)(pa + (((rp * S + s) * 2 + at) * 64 + lane) * 8) = q;
    pidx[((rp * S + s) * 64 + lane) * 2 + at] = (unsigned short)idx;
  }
  // pcol: one thread per (rp, s, h, kq, table): the four staged-row offsets of the lane class (h, kq).
  // Load m of the B operand covers block blk(m, h) = 4*(m/2) + 2*h + (m%2) of the step.
  const int64_t ncol_items = Rp * S * 8 * NT;
  if (gid < ncol_items) {
    const int t = (int)(gid % NT);
    const int64_t g2 = gid / NT;
    const int kq = (int)(g2 & 3), h = (int)((g2 >> 2) & 1);
    const int64_t rs = g2 >> 3;
    const int64_t s = rs % S, rp = rs / S;
    const int64_t r = (rp * 64 + t * 32) / V;     // row block of the pattern that owns this table
    unsigned o = 0;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int blk = 4 * (m >> 1) + 2 * h + (m & 1);
      const int64_t b = s * 8 + blk;
      const unsigned c = (b < B && r < R) ? colidx[(r * B + b) * 4 + kq] : (unsigned)kq;
      o |= (unsigned)(blk * M + c) << (8 * m);
    }
    ((unsigned*)pcol)[gid] = o;
  }
}

int launch_pack(const void* values, const void* meta, const void* colidx, const Dims& d,
                void* packed, hipStream_t st) {
  const PackedLayout pl = packed_layout(d);
  if (pl.total == 0) return VNM_ERR_UNSUPPORTED;
  const int64_t Rp = packed_row_blocks(d);
  const int64_t total = Rp * d.S * 2 * 64;
  char* p = (char*)packed;
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     (const unsigned short*)values, (const unsigned char*)meta,
                     (const unsigned char*)colidx, d.V, d.M, d.R, Rp, d.B, d.S,
                     (unsigned short*)(p + pl.pa_off), (unsigned short*)(p + pl.pidx_off),
                     (unsigned char*)(p + pl.pcol_off));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "pack_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

// ---------------------------------------------------------------- generic spmm
// One thread per output Y[t, o], written straight from the formula on the canonical triple.
// Slow; it is the fallback for shapes the matrix-core kernel does not take and the cross-check
// for that kernel.
template <typename OutT>
__global__ void __launch_bounds__(256)
spmm_generic_kernel(const _Float16* __restrict__ X, int64_t T, int64_t ldx,
                    const _Float16* __restrict__ values, const unsigned char* __restrict__ meta,
                    const unsigned char* __restrict__ colidx, int64_t out, int64_t in, int V, int M,
                    int64_t B, OutT* __restrict__ Y, int64_t ldy, const _Float16* __restrict__ bias,
                    const int* __restrict__ perm_in, const int* __restrict__ perm_out) {
  const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t t = blockIdx.y;
  if (o >= out) return;
  const int64_t r = o / V;
  const _Float16* xrow = X + t * ldx;
  const _Float16* vrow = values + o * 2 * B;
  const unsigned char* mrow = meta + o * ((B + 1) / 2);
  const unsigned char* crow = colidx + r * B * 4;
  float acc = 0.f;
  for (int64_t b = 0; b < B; ++b) {
    const unsigned byte = mrow[b >> 1];
    const unsigned nib = (b & 1) ? (byte >> 4) : (byte & 15u);
    const int64_t c0 = b * M + crow[b * 4 + (nib & 3)];
    const int64_t c1 = b * M + crow[b * 4 + (nib >> 2)];
    // Eq. 6, P_i^T: column c of the weight multiplies input channel perm_in[c]
    const int64_t s0 = (c0 < in) ? (perm_in ? (int64_t)perm_in[c0] : c0) : -1;
    const int64_t s1 = (c1 < in) ? (perm_in ? (int64_t)perm_in[c1] : c1) : -1;
    const float x0 = (s0 >= 0 && s0 < in) ? (float)xrow[s0] : 0.f;
    const float x1 = (s1 >= 0 && s1 < in) ? (float)xrow[s1] : 0.f;
    acc = fmaf((float)vrow[2 * b], x0, acc);
    acc = fmaf((float)vrow[2 * b + 1], x1, acc);
  }
  if (bias) acc += (float)bias[o];
  const int64_t dst = perm_out ? (int64_t)perm_out[o] : o;                  // Eq. 6, P_o^T
  if (dst >= 0 && dst < out) Y[t * ldy + dst] = (OutT)acc;
}

int launch_spmm_generic(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                        const void* colidx, const Dims& d, void* Y, int64_t ldy, int y_dtype,
                        const Fused& f, hipStream_t st) {
  const unsigned gx = (unsigned)((d.out + 255) / 256);
  for (int64_t t0 = 0; t0 < T; t0 += 65535) {                    // grid.y limit
    const int64_t nt = T - t0 < 65535 ? T - t0 : 65535;
    const _Float16* Xs = (const _Float16*)X + t0 * ldx;
    if (y_dtype == 0)
      hipLaunchKernelGGL(spmm_generic_kernel<_Float16>, dim3(gx, (unsigned)nt), dim3(256), 0, st, Xs,
                         nt, ldx, (const _Float16*)values, (const unsigned char*)meta,
                         (const unsigned char*)colidx, d.out, d.in, d.V, d.M, d.B,
                         (_Float16*)Y + t0 * ldy, ldy, f.bias, f.perm_in, f.perm_out);
    else
      hipLaunchKernelGGL(spmm_generic_kernel<float>, dim3(gx, (unsigned)nt), dim3(256), 0, st, Xs,
                         nt, ldx, (const _Float16*)values, (const unsigned char*)meta,
                         (const unsigned char*)colidx, d.out, d.in, d.V, d.M, d.B,
                         (float*)Y + t0 * ldy, ldy, f.bias, f.perm_in, f.perm_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_hip_error(e, "spmm_generic_kernel"); return VNM_ERR_HIP; }
  }
  return VNM_OK;
}

}  // namespace vnm
