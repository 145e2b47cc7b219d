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
//
// GATHER: an input-channel permutation (Section 4.2, Eq. 6: the factor P_i^T applied to X) is folded
// into this pass, which copies every element anyway: image row c of K step s takes column
// perm[8 M s + c] of X, fetched with 2-byte loads (a permutation of the channels leaves nothing
// contiguous in a token's row).
template <int kStageKC, bool GATHER>
__global__ void __launch_bounds__(256)
stage_x_kernel(const unsigned short* __restrict__ X, int64_t T, int64_t ldx, int64_t in, int M,
               int64_t S, int64_t image_bytes, int n_sub, const int* __restrict__ perm,
               unsigned char* __restrict__ Xs) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // column ranges vary fastest over the grid: workgroups that run together then read whole rows of X
  // between them instead of the same 640-byte window of many rows (rows of 8 KiB put such windows on
  // half of the memory channels); 3-6 % on operands that come from HBM
  const int64_t tile = blockIdx.y;
  const int64_t sub0 = (int64_t)blockIdx.x * n_sub;
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
        if (!GATHER) {
          if (t0 + tok < T && col0 + ch * 8 < in) w[i] = *(const uint4*)(X + (t0 + tok) * ldx + col0 + ch * 8);
        } else if (t0 + tok < T && col0 + ch * 8 < in) {               // in % 8 == 0: all 8 entries exist
          const int4 p0 = *(const int4*)(perm + col0 + ch * 8), p1 = *(const int4*)(perm + col0 + ch * 8 + 4);
          const int pc[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
          const unsigned short* xr = X + (t0 + tok) * ldx;
          unsigned h[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) h[e] = (unsigned)pc[e] < (unsigned)in ? xr[pc[e]] : 0u;   // (in < 2^31)
          w[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        }
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
    // item = (column c, token octet tq): a wave takes 8 octets x 8 columns, so that its 2-byte reads of a
    // tile whose rows are an odd number of dwords apart fall into 32 different banks (the two columns of
    // a dword share an address) and its stores are whole 128-byte lines; combination number
    // wave + 4 i picks the half of the octets and the group of 8 columns
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (i < NI) {
        const int comb = (tid >> 6) + 4 * i;
        const int tq = (comb & 1) * 8 + (tid & 7), c = (comb >> 1) * 8 + ((tid >> 3) & 7);
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

// Channel permutation of the rows of a token-major matrix (Section 4.2, Eq. 6), one workgroup per
// token row, the whole row passing through LDS so that both the global reads and the global writes
// are contiguous and only the LDS accesses are scattered:
//   SCATTER = false:  dst[t, j] = src[t, idx[j]]      (P_i^T applied to X; an entry of idx outside
//                                                      0..n-1 gives 0)
//   SCATTER = true:   dst[t, idx[j]] = src[t, j]      (P_o^T applied to Y; an entry outside the range
//                                                      is dropped, columns nothing maps to become 0)
// dst may be src (each workgroup reads its whole row before it writes any of it).
// VEC: 16-byte global accesses (n a multiple of 16 / sizeof(E), rows 16-byte aligned).
// The gather form may split a row's destination over gridDim.y workgroups (each reads the whole
// source row, which then comes from L2): few rows alone would leave most of the chip idle.
template <typename E, bool SCATTER, bool VEC>
__global__ void __launch_bounds__(256)
permute_rows_kernel(const E* __restrict__ src, int64_t ld_src, E* dst, int64_t ld_dst, int64_t n,
                    const int* __restrict__ idx) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  E* row = (E*)smem;
  constexpr int EPV = 16 / (int)sizeof(E);             // elements per 16-byte vector
  const int64_t t = blockIdx.x;
  const E* s = src + t * ld_src;
  E* d = dst + t * ld_dst;
  const int tid = threadIdx.x;
  if (SCATTER) {
    if (VEC) {
      const int64_t nv = n / EPV;
      for (int64_t v = tid; v < nv; v += 256) ((uint4*)row)[v] = make_uint4(0, 0, 0, 0);
      __syncthreads();
      for (int64_t v = tid; v < nv; v += 256) {
        const uint4 w = ((const uint4*)s)[v];
        const E* e = (const E*)&w;
        int k[EPV];
#pragma unroll
        for (int q = 0; q < EPV / 4; ++q) *(int4*)(k + 4 * q) = ((const int4*)idx)[v * (EPV / 4) + q];
#pragma unroll
        for (int q = 0; q < EPV; ++q)
          if ((unsigned)k[q] < (unsigned)n) row[k[q]] = e[q];
      }
      __syncthreads();
      for (int64_t v = tid; v < nv; v += 256) ((uint4*)d)[v] = ((const uint4*)row)[v];
    } else {
      for (int64_t j = tid; j < n; j += 256) row[j] = (E)0;
      __syncthreads();
      for (int64_t j = tid; j < n; j += 256) {
        const int k = idx[j];
        const E v = s[j];
        if ((unsigned)k < (unsigned)n) row[k] = v;
      }
      __syncthreads();
      for (int64_t j = tid; j < n; j += 256) d[j] = row[j];
    }
  } else {
    // destination range of this workgroup
    const int64_t per = ((n + gridDim.y - 1) / gridDim.y + EPV - 1) / EPV * EPV;
    const int64_t j0 = (int64_t)blockIdx.y * per, j1 = j0 + per < n ? j0 + per : n;
    if (VEC) {
      const int64_t nv = n / EPV;
      for (int64_t v = tid; v < nv; v += 256) ((uint4*)row)[v] = ((const uint4*)s)[v];
      __syncthreads();
      for (int64_t v = j0 / EPV + tid; v < j1 / EPV; v += 256) {
        int k[EPV];
#pragma unroll
        for (int q = 0; q < EPV / 4; ++q) *(int4*)(k + 4 * q) = ((const int4*)idx)[v * (EPV / 4) + q];
        uint4 w;
        E* e = (E*)&w;
#pragma unroll
        for (int q = 0; q < EPV; ++q) e[q] = (unsigned)k[q] < (unsigned)n ? row[k[q]] : (E)0;
        ((uint4*)d)[v] = w;
      }
    } else {
      for (int64_t j = tid; j < n; j += 256) row[j] = s[j];
      __syncthreads();
      for (int64_t j = j0 + tid; j < j1; j += 256) {
        const int k = idx[j];
        d[j] = (unsigned)k < (unsigned)n ? row[k] : (E)0;
      }
    }
  }
}

int64_t permute_rows_max_bytes() { return 144 * 1024; }

template <typename E, bool SCATTER, bool VEC>
static int launch_permute_cfg(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t T, int64_t n,
                              const int* idx, hipStream_t st) {
  auto kern = permute_rows_kernel<E, SCATTER, VEC>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(permute_rows)")) return rc_lds;
  // gather form: split rows until about two workgroups per CU exist
  int64_t ny = 1;
  if (!SCATTER && T < 512) { ny = 512 / T; if (ny > 16) ny = 16; if (ny * 2048 > n) ny = n / 2048 > 0 ? n / 2048 : 1; }
  hipLaunchKernelGGL(kern, dim3((unsigned)T, (unsigned)ny), dim3(256), (size_t)n * sizeof(E), st, (const E*)src,
                     ld_src, (E*)dst, ld_dst, n, idx);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "permute_rows_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

template <typename E>
static int launch_permute_e(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t T, int64_t n,
                            bool scatter, const int* idx, hipStream_t st) {
  const int64_t epv = 16 / (int64_t)sizeof(E);
  const bool vec = n % epv == 0 && ld_src % epv == 0 && ld_dst % epv == 0 && (((uintptr_t)src | (uintptr_t)dst | (uintptr_t)idx) & 15) == 0;
  if (scatter)
    return vec ? launch_permute_cfg<E, true, true>(src, ld_src, dst, ld_dst, T, n, idx, st)
               : launch_permute_cfg<E, true, false>(src, ld_src, dst, ld_dst, T, n, idx, st);
  return vec ? launch_permute_cfg<E, false, true>(src, ld_src, dst, ld_dst, T, n, idx, st)
             : launch_permute_cfg<E, false, false>(src, ld_src, dst, ld_dst, T, n, idx, st);
}

int launch_permute_rows(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t T, int64_t n,
                        int elem_bytes, bool scatter, const int* idx, hipStream_t st) {
  if (T > 0x7FFFFFFF || n * elem_bytes > permute_rows_max_bytes()) return VNM_ERR_UNSUPPORTED;
  if (elem_bytes == 2) return launch_permute_e<unsigned short>(src, ld_src, dst, ld_dst, T, n, scatter, idx, st);
  return launch_permute_e<unsigned>(src, ld_src, dst, ld_dst, T, n, scatter, idx, st);
}

int64_t staged_bytes(int64_t T, const Dims& d) {
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  // + 3 images that the product kernel's look-ahead copies may read (never use) past the last tile
  return (tiles * d.S + 3) * image_bytes(d.M);
}

template <int KC, bool GATHER>
static int launch_stage_cfg(const void* X, int64_t T, int64_t ldx, const Dims& d, const int* perm, void* Xs,
                            dim3 grid, size_t lds, int n_sub, hipStream_t st) {
  auto kern = stage_x_kernel<KC, GATHER>;
  if (int rc_lds = allow_big_lds((const void*)kern, "hipFuncSetAttribute(stage_x)")) return rc_lds;
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const unsigned short*)X, T, ldx, d.in, d.M, d.S,
                     image_bytes(d.M), n_sub, perm, (unsigned char*)Xs);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error(e, "stage_x_kernel"); return VNM_ERR_HIP; }
  return VNM_OK;
}

int launch_stage_x(const void* X, int64_t T, int64_t ldx, const Dims& d, const int* perm_in, void* Xs,
                   hipStream_t st) {
  const int64_t tiles = (T + kTokTile - 1) / kTokTile;
  // K steps per sub-chunk: 4 (rows of 64 M bytes per load) while a thread's share fits 16 registers sets
  const int KC = d.M <= 8 ? 4 : 2;
  const int64_t subs = (d.S + KC - 1) / KC;
  // two sub-chunks per workgroup (one level of read/write overlap measured best) unless that
  // would leave fewer workgroups than CUs
  int64_t n_sub = tiles * subs >= 512 ? 2 : 1;
  const int64_t gy = (subs + n_sub - 1) / n_sub;
  if (gy > 0x7FFFFFFF || tiles > 65535) return VNM_ERR_UNSUPPORTED;
  const size_t lds = (size_t)kTokTile * (KC * d.M * 16 + 4);
  dim3 grid((unsigned)gy, (unsigned)tiles);
  if (KC == 4)
    return perm_in ? launch_stage_cfg<4, true>(X, T, ldx, d, perm_in, Xs, grid, lds, (int)n_sub, st)
                   : launch_stage_cfg<4, false>(X, T, ldx, d, nullptr, Xs, grid, lds, (int)n_sub, st);
  return perm_in ? launch_stage_cfg<2, true>(X, T, ldx, d, perm_in, Xs, grid, lds, (int)n_sub, st)
                 : launch_stage_cfg<2, false>(X, T, ldx, d, nullptr, Xs, grid, lds, (int)n_sub, st);
}

}  // namespace vnm
