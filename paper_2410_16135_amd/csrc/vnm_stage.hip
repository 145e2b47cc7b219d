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

// One workgroup: one token tile x a run of sub-chunks of kStageKC K steps each.  Per sub-chunk,
// rows of X are read with 16-byte loads (lanes along the columns) and parked in an LDS tile
// [token][column]; the tile is read back column-wise and written 16 bytes (8 tokens of one column)
// per lane, 16 lanes per image row.  The loads of the next sub-chunk are issued before the stores
// of the current one, so that reads and writes of HBM overlap inside every workgroup.
template <int kStageKC>
__global__ void __launch_bounds__(256)
stage_x_kernel(const unsigned short* __restrict__ X, int64_t T, int64_t ldx, int64_t in, int M,
               int64_t S, int64_t image_bytes, int n_sub, unsigned char* __restrict__ Xs) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int64_t tile = blockIdx.x;
  const int64_t sub0 = (int64_t)blockIdx.y * n_sub;
  const int64_t t0 = tile * kTokTile;
  const int CH = kStageKC * M;                         // 16-byte chunks per token row and sub-chunk
  const int pitch = CH * 16 + 4;                       // bytes; odd number of dwords
  const int tid = threadIdx.x;
  // item i of this thread is (token, chunk) number tid + 256 i in row-major order: NI items each
  const int NI = kStageKC * M / 2;
  const int tok_first = tid / CH, ch_first = tid - tok_first * CH;
  const int dtok = 256 / CH, dch = 256 - dtok * CH;
  uint4 w[16];
  auto load = [&](int64_t sub) {
    const int64_t col0 = sub * kStageKC * 8 * M;
    int tok = tok_first, ch = ch_first;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (i < NI) {
        w[i] = make_uint4(0, 0, 0, 0);
        if (t0 + tok < T && col0 + ch * 8 < in) w[i] = *(const uint4*)(X + (t0 + tok) * ldx + col0 + ch * 8);
        ch += dch; tok += dtok;
        if (ch >= CH) { ch -= CH; ++tok; }
      }
    }
  };
  if (sub0 * kStageKC < S) load(sub0);
  for (int k = 0; k < n_sub; ++k) {
    const int64_t sub = sub0 + k;
    const int64_t s_begin = sub * kStageKC;
    if (s_begin >= S) break;
    {
      int tok = tok_first, ch = ch_first;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (i < NI) {
          unsigned* d = (unsigned*)(smem + (size_t)tok * pitch + ch * 16);
          d[0] = w[i].x; d[1] = w[i].y; d[2] = w[i].z; d[3] = w[i].w;
          ch += dch; tok += dtok;
          if (ch >= CH) { ch -= CH; ++tok; }
        }
      }
    }
    __syncthreads();
    if (k + 1 < n_sub && (sub + 1) * kStageKC < S) load(sub + 1);
    // item = (column c, token octet tq)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (i < NI) {
        const int tq = tid & 15, c = (tid >> 4) + 16 * i;
        const int ks = kStageKC == 2 ? (c >= 8 * M ? 1 : 0) : c / (8 * M), cr = c - ks * 8 * M;
        if (s_begin + ks < S) {
          const unsigned char* src = smem + (size_t)(tq * 8) * pitch + c * 2;
          unsigned short h[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) h[e] = *(const unsigned short*)(src + (size_t)e * pitch);
          uint4 o;
          o.x = h[0] | ((unsigned)h[1] << 16); o.y = h[2] | ((unsigned)h[3] << 16);
          o.z = h[4] | ((unsigned)h[5] << 16); o.w = h[6] | ((unsigned)h[7] << 16);
          unsigned char* dst = Xs + (tile * S + s_begin + ks) * image_bytes + (size_t)cr * kImagePitch + tq * 16;
          *(uint4*)dst = o;
        }
      }
    }
    __syncthreads();
  }
}

int64_t staged_bytes(int64_t T, const Dims& d) {
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  // + 3 images that the product kernel's look-ahead copies may read (never use) past the last tile
  return (tiles * d.S + 3) * image_bytes(d.M);
}

int launch_stage_x(const void* X, int64_t T, int64_t ldx, const Dims& d, void* Xs, hipStream_t st) {
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  // K steps per sub-chunk: 4 (rows of 64 M bytes per load) while a thread's share fits 16 registers sets
  const int KC = d.M <= 8 ? 4 : 2;
  const int64_t subs = (d.S + KC - 1) / KC;
  // two sub-chunks per workgroup (one level of read/write overlap measured best) unless that
  // would leave fewer workgroups than CUs
  int64_t n_sub = tiles * subs >= 512 ? 2 : 1;
  const int64_t gy = (subs + n_sub - 1) / n_sub;
  if (tiles > 0x7FFFFFFF || gy > 65535) return VNM_ERR_UNSUPPORTED;
  const size_t lds = (size_t)kTokTile * (KC * d.M * 16 + 4);
  if (int rc_lds = allow_big_lds(KC == 4 ? (const void*)stage_x_kernel<4> : (const void*)stage_x_kernel<2>,
                                 "hipFuncSetAttribute(stage_x)")) return rc_lds;
  dim3 grid((unsigned)tiles, (unsigned)gy);
  if (KC == 4)
    hipLaunchKernelGGL(stage_x_kernel<4>, grid, dim3(256), lds, st, (const unsigned short*)X, T, ldx, d.in, d.M,
                       d.S, image_bytes(d.M), (int)n_sub, (unsigned char*)Xs);
  else
    hipLaunchKernelGGL(stage_x_kernel<2>, grid, dim3(256), lds, st, (const unsigned short*)X, T, ldx, d.in, d.M,
                       d.S, image_bytes(d.M), (int)n_sub, (unsigned char*)Xs);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "stage_x_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

}  // namespace vnm
