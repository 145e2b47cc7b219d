// Internal declarations shared by the HIP sources of libvnm (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "vnm.h"

namespace vnm {

// Padded shape of one layer (Section 3, weight padding) plus the tiling of the packed copy.
struct Dims {
  int64_t out, in, out_pad, in_pad;
  int64_t R;       // row blocks
  int64_t B;       // column blocks
  int64_t S;       // K steps of the matrix-core kernel: groups of 8 column blocks (32 compacted K)
  int V, M;
};

// Byte offsets of the three sections of the packed copy.
//   pa   fp16 [R][S][V/32][64 lanes][8]   A operand of smfmac 32x32x32 in lane order
//   pidx u16  [R][S][64 lanes][V/32]      2-bit positions, 16 bits per (lane, 32-row tile)
//   pcol u8   [R][S][2][4][4]             staged-row offsets blk*M + c in B-operand lane order
struct PackedLayout {
  int64_t pa_off, pidx_off, pcol_off, total;
};

inline Dims make_dims(int64_t out, int64_t in, int V, int M) {
  Dims d;
  d.out = out; d.in = in; d.V = V; d.M = M;
  d.R = (out + V - 1) / V;
  d.B = (in + M - 1) / M;
  d.out_pad = d.R * V;
  d.in_pad = d.B * M;
  d.S = (d.B + 7) / 8;
  return d;
}

inline bool has_packed(int V, int M) { return (V == 32 || V == 64 || V == 128) && M <= 16; }

// The matrix-core copy is organised in row blocks of 64 rows (two 32-row tiles) whatever V is: a
// 128-row block of the pattern is stored as two 64-row blocks that carry the same column table, and
// two 32-row blocks of the pattern share one 64-row block that carries both their column tables
// (table t belongs to tile t).  One product kernel then serves V = 32, 64 and 128.
constexpr int kPackedRows = 64;
inline int64_t packed_row_blocks(const Dims& d) { return (d.out_pad + kPackedRows - 1) / kPackedRows; }
inline int packed_tables(int V) { return V == 32 ? 2 : 1; }

inline PackedLayout packed_layout(const Dims& d) {
  PackedLayout p{0, 0, 0, 0};
  if (!has_packed(d.V, d.M)) return p;
  auto up = [](int64_t x) { return (x + 255) / 256 * 256; };
  const int64_t Rp = packed_row_blocks(d);
  p.pa_off = 0;
  p.pidx_off = up(Rp * d.S * 2 * 64 * 8 * 2);
  p.pcol_off = p.pidx_off + up(Rp * d.S * 64 * 2 * 2);
  // + 8 KiB that the product kernel's look-ahead loads may read (never use) past the last row block
  p.total = p.pcol_off + up(Rp * d.S * 32 * packed_tables(d.V)) + 8192;
  return p;
}

// Staged activations (see vnm_stage.hip): token tiles of kTokTile, image rows kImagePitch bytes apart.
constexpr int kTokTile = 128;
constexpr int kImagePitch = kTokTile * 2 + 64;
inline int64_t image_bytes(int M) { return ((int64_t)8 * M * kImagePitch + 1023) / 1024 * 1024; }
int64_t staged_bytes(int64_t T, const Dims& d);

// Optional steps fused around the product (Section 4.2, Eq. 6, plus the layer's bias); all null = the
// plain product.  Entries of a permutation outside its range never fault: such an input column reads
// as zero, such an output channel is not stored.
struct Fused {
  const _Float16* bias = nullptr;   // [out], in the row order of the compressed weight
  const int* perm_in = nullptr;     // [in]:  column i of the weight multiplies X[:, perm_in[i]]
  const int* perm_out = nullptr;    // [out]: row o of the weight produces Y[:, perm_out[o]]
  bool any_out() const { return bias || perm_out; }
};

void set_hip_error(hipError_t e, const char* where);
void set_error_text(const char* text);           // what vnm_last_hip_error() returns next (calling thread)
// Host-side argument checks shared by the entry points (vnm_api.hip, no device code in that file)
int check_pattern(int64_t out, int64_t in, int V, int N, int M);
constexpr int kProceed = -1;                     // spmm_validate: arguments are fine and there is work to enqueue
int spmm_validate(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta, const void* colidx,
                  const void* packed, int64_t out, int64_t in, int V, int N, int M, const struct Fused& f,
                  const void* Y, int64_t ldy, int y_dtype, int path, int64_t workspace_bytes);
int spmm_impl(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta, const void* colidx,
              const void* packed, int64_t out, int64_t in, int V, int N, int M, const struct Fused& f, void* Y,
              int64_t ldy, int y_dtype, int path, void* workspace, int64_t workspace_bytes, void* stream);
// Raises a kernel's dynamic-LDS limit to the 160 KiB of a gfx950 CU, once per (kernel, device); thread-safe.
// Returns a vnm_status.
int allow_big_lds(const void* kernel, const char* what);

// launchers (each returns a vnm_status)
int launch_prune_compress(const void* W, int64_t ldw, const Dims& d, void* values, void* meta,
                          void* colidx, void* mask, hipStream_t st);
bool prune_fast_applicable(const void* W, int64_t ldw, const Dims& d, const void* mask);
int launch_prune_fast(const void* W, int64_t ldw, const Dims& d, void* values, void* meta, void* colidx,
                      void* mask, void* packed, hipStream_t st);
bool prune_fast_scored_applicable(const void* W, int64_t ldw, const void* S, int64_t lds_s, const Dims& d);
int launch_prune_fast_scored(const void* W, int64_t ldw, const void* S, int64_t lds_s, const Dims& d, void* values,
                             void* meta, void* colidx, void* mask, void* packed, hipStream_t st);
bool decompress_fast_applicable(const void* W_out, int64_t ldw, const Dims& d);
int launch_decompress_fast(const void* values, const void* meta, const void* colidx, const Dims& d,
                           void* W_out, int64_t ldw, hipStream_t st);
int launch_pack(const void* values, const void* meta, const void* colidx, const Dims& d,
                void* packed, hipStream_t st);
int launch_decompress(const void* values, const void* meta, const void* colidx, const Dims& d,
                      void* W_out, int64_t ldw, hipStream_t st);
int launch_spmm_generic(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                        const void* colidx, const Dims& d, void* Y, int64_t ldy, int y_dtype,
                        const Fused& f, hipStream_t st);
// perm_in (or null): image row c of K step s holds X[:, perm_in[8 M s + c]]
int launch_stage_x(const void* X, int64_t T, int64_t ldx, const Dims& d, const int* perm_in, void* Xs,
                   hipStream_t st);
// Row-wise channel permutation through LDS: gather (dst[t, j] = src[t, idx[j]]) or scatter
// (dst[t, idx[j]] = src[t, j], in place allowed); rows of n elements of 2 or 4 bytes, at most
// permute_rows_max_bytes() per row.
int64_t permute_rows_max_bytes();
int launch_permute_rows(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t T, int64_t n,
                        int elem_bytes, bool scatter, const int* idx, hipStream_t st);
bool spmm_smfmac_applicable(const void* X, int64_t ldx, const Dims& d);
// Importance scores other than |w| (vnm_score.hip)
int launch_ria_scores(const void* W, int64_t out, int64_t in, int64_t ldw, const void* act, void* S,
                      int64_t lds, void* workspace, hipStream_t st);
int launch_prune_scored(const void* W, int64_t ldw, const void* S, int64_t lds, const Dims& d, void* values,
                        void* meta, void* colidx, void* mask, hipStream_t st);
// Wm = fp16(W + scale * B A) in a fixed fp32 order (vnm_score.hip)
int launch_lora_merge(const void* W, int64_t ldw, const void* B, int64_t ldb, const void* A, int64_t lda, int r,
                      float scale, int64_t out, int64_t in, void* Wm, int64_t ldm, hipStream_t st);
// Single-kernel product for at most skinny_max_tokens() tokens, straight from X (no staging, no workspace).
int64_t skinny_max_tokens();
// The same kernels also serve up to 256 tokens where their workgroups fit the compute units at once (no
// staging; scratch_bytes: what the caller can offer for split-K partial products).
bool skinny_groups_applicable(int64_t T, const Dims& d, int64_t scratch_bytes);
int launch_spmm_skinny(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                       void* Y, int64_t ldy, int y_dtype, void* scratch, int64_t scratch_bytes,
                       const Fused& f, hipStream_t st);
// Product for at most gemv_max_tokens() tokens on the vector ALUs (vnm_spmm_gemv.hip): the packed weight
// streamed once, no matrix instructions, no workspace.  X as for the few-token kernels.
int64_t gemv_max_tokens();
bool spmm_gemv_applicable(int64_t T, int64_t ldx, const Dims& d);
int launch_spmm_gemv(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                     void* Y, int64_t ldy, int y_dtype, const Fused& f, hipStream_t st);
// Single-kernel product without a staging pass (vnm_spmm_resident.hip): the workgroup's slice of X
// is turned around into LDS by the kernel itself; for a K range that fits LDS, or few enough
// output channels for K to stream through LDS in chunks.
bool spmm_resident_applicable(int64_t T, const Dims& d);
int launch_spmm_resident(const void* X, int64_t T, int64_t ldx, const void* packed, const Dims& d,
                         void* Y, int64_t ldy, int y_dtype, const Fused& f, hipStream_t st);
// Y = sum of KS fp32 partial products [KS][T][out] held in `part` (+ bias, output permutation)
int launch_splitk_reduce(const void* part, int KS, int64_t T, int64_t out, void* Y, int64_t ldy,
                         int y_dtype, const Fused& f, hipStream_t st);
// Split-K scratch of the product kernel for small token counts (fp32 partial products), 0 when unused.
int64_t splitk_scratch_bytes(int64_t T, int64_t out);
// f.perm_in is not this kernel's business (it is applied when X is staged)
int launch_spmm_smfmac(const void* Xs, int64_t T, const void* packed, const Dims& d,
                       void* Y, int64_t ldy, int y_dtype, void* scratch, int64_t scratch_bytes,
                       const Fused& f, hipStream_t st);

}  // namespace vnm
