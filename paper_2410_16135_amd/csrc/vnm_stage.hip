// Staging pass of vnm_spmm: X [T x in] (row-major, token-major) is re-laid once per call into the
// order the matrix-core kernel streams it in, so that every workgroup of that kernel can fetch its
// operand with plain linear, fully coalesced asynchronous copies into LDS.
//
// Staged layout: one IMAGE per (token tile of 128, K step of 8 column blocks):
//     image[row c][token]   c = 0 .. 8*M-1 (raw input columns of the K step), 128 tokens, fp16,
// rows kImagePitch bytes apart (256 data bytes + 64 pad bytes, so that rows M apart fall into
// different LDS bank groups when the kernel gathers 4 rows per block), the image itself padded to a
// multiple of 1 KiB (one wave-wide 16-byte-per-lane copy).  Tokens beyond T and columns beyond `in`
// are zero.  Transposing here -- once per element -- instead of inside the product kernel -- once
// per element per group of row blocks -- is what keeps the product kernel's inner loop free of
// shuffles and of scattered 16-byte loads.
#include "vnm_internal.h"

namespace vnm {

// One workgroup: 128 tokens x (KG K steps).  Phase 1 reads rows of X with 16-byte loads (lanes along
// the columns) into an LDS tile [token][column]; phase 2 reads it back column-wise and writes 16
// bytes (8 tokens of one column) per lane, 16 lanes per image row.
constexpr int kStageKG = 4;

__global__ void __launch_bounds__(256)
stage_x_kernel(const unsigned short* __restrict__ X, int64_t T, int64_t ldx, int64_t in, int M,
               int64_t S, int64_t image_bytes, unsigned char* __restrict__ Xs) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int64_t tile = blockIdx.x;
  const int64_t s_begin = (int64_t)blockIdx.y * kStageKG;
  const int nks = (int)((S - s_begin) < kStageKG ? (S - s_begin) : kStageKG);
  const int ncol = nks * 8 * M;                 // columns of this workgroup (multiple of 8)
  const int64_t col0 = s_begin * 8 * M;
  const int64_t t0 = tile * kTokTile;
  const int pitch = ncol * 2 + 4;               // bytes; 4-byte aligned, odd number of dwords
  const int tid = threadIdx.x;
  // phase 1
  const int chunks = ncol / 8;                  // 16-byte chunks per token row
  for (int item = tid; item < kTokTile * chunks; item += 256) {
    const int tok = item / chunks, ch = item - tok * chunks;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (t0 + tok < T && col0 + ch * 8 < in) v = *(const uint4*)(X + (t0 + tok) * ldx + col0 + ch * 8);
    unsigned* d = (unsigned*)(smem + (size_t)tok * pitch + ch * 16);
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
  }
  __syncthreads();
  // phase 2: item = (column c, token octet tq)
  for (int item = tid; item < ncol * 16; item += 256) {
    const int tq = item & 15, c = item >> 4;
    const unsigned char* src = smem + (size_t)(tq * 8) * pitch + c * 2;
    unsigned short h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) h[i] = *(const unsigned short*)(src + (size_t)i * pitch);
    uint4 o;
    o.x = h[0] | ((unsigned)h[1] << 16); o.y = h[2] | ((unsigned)h[3] << 16);
    o.z = h[4] | ((unsigned)h[5] << 16); o.w = h[6] | ((unsigned)h[7] << 16);
    const int ks = c / (8 * M), cr = c - ks * 8 * M;
    unsigned char* dst = Xs + (tile * S + s_begin + ks) * image_bytes + (size_t)cr * kImagePitch + tq * 16;
    *(uint4*)dst = o;
  }
}

int64_t staged_bytes(int64_t T, const Dims& d) {
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  // + 3 images that the product kernel's look-ahead copies may read (never use) past the last tile
  return (tiles * d.S + 3) * image_bytes(d.M);
}

int launch_stage_x(const void* X, int64_t T, int64_t ldx, const Dims& d, void* Xs, hipStream_t st) {
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  if (tiles > 0x7FFFFFFF || (d.S + kStageKG - 1) / kStageKG > 65535) return VNM_ERR_UNSUPPORTED;
  const size_t lds = (size_t)kTokTile * (kStageKG * 8 * d.M * 2 + 4);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)stage_x_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) { set_hip_error(e, "hipFuncSetAttribute(stage_x)"); return VNM_ERR_HIP; }
    attr_set = true;
  }
  dim3 grid((unsigned)tiles, (unsigned)((d.S + kStageKG - 1) / kStageKG));
  hipLaunchKernelGGL(stage_x_kernel, grid, dim3(256), lds, st, (const unsigned short*)X, T, ldx, d.in, d.M,
                     d.S, image_bytes(d.M), (unsigned char*)Xs);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "stage_x_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
