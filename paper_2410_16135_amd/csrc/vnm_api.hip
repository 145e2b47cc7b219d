// C ABI of libvnm: argument validation on the host, then dispatch to the kernel launchers.
#include <string.h>
#include <stdio.h>
#include <mutex>
#include <set>
#include <utility>
#include <vector>
#include "vnm_internal.h"

namespace vnm {
static thread_local char g_hip_error[256] = "";
void set_hip_error(hipError_t e, const char* where) {
  snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", where, hipGetErrorString(e));
}
void set_error_text(const char* text) { snprintf(g_hip_error, sizeof(g_hip_error), "%s", text); }

int allow_big_lds(const void* kernel, const char* what) {
  static std::mutex mu;
  static std::set<std::pair<const void*, int>> done;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_hip_error(e, "hipGetDevice"); return VNM_ERR_HIP; }
  std::lock_guard<std::mutex> lock(mu);
  if (done.count({kernel, dev})) return VNM_OK;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e != hipSuccess) { set_hip_error(e, what); return VNM_ERR_HIP; }
  done.insert({kernel, dev});
  return VNM_OK;
}
}  // namespace vnm

using namespace vnm;

int vnm::check_pattern(int64_t out, int64_t in, int V, int N, int M) {
  if (out <= 0 || in <= 0) return VNM_ERR_SHAPE;
  if (N != 2) return VNM_ERR_UNSUPPORTED;                       // Section 4.1: N is always 2
  if (M < 4 || M > 255) return VNM_ERR_UNSUPPORTED;             // colidx is a byte
  if (!(V == 16 || V == 32 || V == 64 || V == 128)) return VNM_ERR_UNSUPPORTED;
  return VNM_OK;
}

extern "C" int vnm_query_sizes(int64_t out, int64_t in, int V, int N, int M, vnm_sizes* s) {
  if (!s) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  Dims d = make_dims(out, in, V, M);
  s->out_pad = d.out_pad;
  s->in_pad = d.in_pad;
  s->row_blocks = d.R;
  s->col_blocks = d.B;
  s->kc = 4 * d.B;
  s->values_elems = d.out_pad * 2 * d.B;
  s->meta_bytes = d.out_pad * ((d.B + 1) / 2);
  s->colidx_bytes = d.R * d.B * 4;
  s->packed_bytes = packed_layout(d).total;
  s->workspace_bytes = 0;
  return VNM_OK;
}

extern "C" int vnm_prune_compress(const void* W, int64_t out, int64_t in, int64_t ldw, int V, int N,
                                  int M, void* values, void* meta, void* colidx, void* mask,
                                  void* packed, void* workspace, int64_t workspace_bytes,
                                  void* stream) {
  (void)workspace;
  if (!W || !values || !meta || !colidx) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (ldw < in) return VNM_ERR_SHAPE;
  if (workspace_bytes < 0) return VNM_ERR_WORKSPACE;
  if (((uintptr_t)W & 1) || ((uintptr_t)values & 3)) return VNM_ERR_ALIGN;
  Dims d = make_dims(out, in, V, M);
  if (packed) {
    if (!has_packed(V, M)) return VNM_ERR_UNSUPPORTED;
    if ((uintptr_t)packed & 255) return VNM_ERR_ALIGN;
  }
  hipStream_t st = (hipStream_t)stream;
  if (prune_fast_applicable(W, ldw, d, mask) && ((uintptr_t)colidx & 3) == 0 && (!packed || has_packed(V, M)))
    return launch_prune_fast(W, ldw, d, values, meta, colidx, mask, packed, st);
  rc = launch_prune_compress(W, ldw, d, values, meta, colidx, mask, st);
  if (rc) return rc;
  if (packed) rc = launch_pack(values, meta, colidx, d, packed, st);
  return rc;
}

extern "C" int vnm_ria_scores(const void* W, int64_t out, int64_t in, int64_t ldw, const void* act,
                              void* S, int64_t lds, void* workspace, int64_t workspace_bytes,
                              void* stream) {
  if (!W || !act || !S || !workspace) return VNM_ERR_NULL;
  if (out <= 0 || in <= 0 || ldw < in || lds < in) return VNM_ERR_SHAPE;
  if (workspace_bytes < (out + in) * 8) return VNM_ERR_WORKSPACE;
  if (((uintptr_t)W & 1) || ((uintptr_t)act & 3) || ((uintptr_t)S & 3) || ((uintptr_t)workspace & 7)) return VNM_ERR_ALIGN;
  return launch_ria_scores(W, out, in, ldw, act, S, lds, workspace, (hipStream_t)stream);
}

extern "C" int vnm_prune_compress_scored(const void* W, const void* S, int64_t out, int64_t in,
                                         int64_t ldw, int64_t lds, int V, int N, int M, void* values,
                                         void* meta, void* colidx, void* mask, void* packed,
                                         void* stream) {
  if (!W || !S || !values || !meta || !colidx) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (ldw < in || lds < in) return VNM_ERR_SHAPE;
  if (((uintptr_t)W & 1) || ((uintptr_t)S & 3) || ((uintptr_t)values & 3) || ((uintptr_t)colidx & 3)) return VNM_ERR_ALIGN;
  const Dims d = make_dims(out, in, V, M);
  if (packed) {
    if (!has_packed(V, M)) return VNM_ERR_UNSUPPORTED;
    if ((uintptr_t)packed & 255) return VNM_ERR_ALIGN;
  }
  hipStream_t st = (hipStream_t)stream;
  // one pass with the weight and score tiles in LDS, packed copy included, where shape and alignment allow
  if (prune_fast_scored_applicable(W, ldw, S, lds, d) && (!packed || has_packed(V, M)))
    return launch_prune_fast_scored(W, ldw, S, lds, d, values, meta, colidx, mask, packed, st);
  rc = launch_prune_scored(W, ldw, S, lds, d, values, meta, colidx, mask, st);
  if (rc) return rc;
  if (packed) return launch_pack(values, meta, colidx, d, packed, st);
  return VNM_OK;
}

extern "C" int vnm_lora_merge(const void* W, int64_t out, int64_t in, int64_t ldw, const void* B, int64_t ldb,
                              const void* A, int64_t lda, int r, float scale, void* W_merged, int64_t ldm,
                              void* stream) {
  if (!W || !W_merged || (r > 0 && (!B || !A))) return VNM_ERR_NULL;
  if (out <= 0 || in <= 0 || r < 0 || ldw < in || ldm < in || (r > 0 && (ldb < r || lda < in))) return VNM_ERR_SHAPE;
  if (((uintptr_t)W & 1) || ((uintptr_t)W_merged & 1) || ((uintptr_t)B & 3) || ((uintptr_t)A & 3)) return VNM_ERR_ALIGN;
  return launch_lora_merge(W, ldw, B, ldb, A, lda, r, scale, out, in, W_merged, ldm, (hipStream_t)stream);
}

extern "C" int vnm_pack(const void* values, const void* meta, const void* colidx, int64_t out,
                        int64_t in, int V, int N, int M, void* packed, void* stream) {
  if (!values || !meta || !colidx || !packed) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (!has_packed(V, M)) return VNM_ERR_UNSUPPORTED;
  if ((uintptr_t)packed & 255) return VNM_ERR_ALIGN;
  if ((uintptr_t)values & 3) return VNM_ERR_ALIGN;
  return launch_pack(values, meta, colidx, make_dims(out, in, V, M), packed, (hipStream_t)stream);
}

// Host-side argument checks of vnm_spmm and its variants; nothing here touches the device.
// Returns a vnm_status, or kProceed when there is work to enqueue.
int vnm::spmm_validate(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                         const void* colidx, const void* packed, int64_t out, int64_t in, int V, int N, int M,
                         const Fused& f, const void* Y, int64_t ldy, int y_dtype, int path, int64_t workspace_bytes) {
  if (!values || !meta || !colidx) return VNM_ERR_NULL;
  if (T != 0 && (!X || !Y)) return VNM_ERR_NULL;                 // an empty batch may come with null X, Y
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (T < 0 || ldx < in || ldy < out) return VNM_ERR_SHAPE;
  if (y_dtype != 0 && y_dtype != 1) return VNM_ERR_UNSUPPORTED;
  if (path != VNM_PATH_AUTO && path != VNM_PATH_GENERIC && path != VNM_PATH_SMFMAC)
    return VNM_ERR_UNSUPPORTED;
  if (workspace_bytes < 0) return VNM_ERR_WORKSPACE;
  if (((uintptr_t)X & 1) || ((uintptr_t)values & 3)) return VNM_ERR_ALIGN;
  if ((uintptr_t)Y & (y_dtype == 0 ? 1 : 3)) return VNM_ERR_ALIGN;
  if (packed && ((uintptr_t)packed & 255)) return VNM_ERR_ALIGN;
  if (((uintptr_t)f.bias & 1) || ((uintptr_t)f.perm_in & 15) || ((uintptr_t)f.perm_out & 3)) return VNM_ERR_ALIGN;
  if (T == 0) return VNM_OK;
  const Dims d = make_dims(out, in, V, M);
  if (path == VNM_PATH_SMFMAC && !(packed && has_packed(V, M) && spmm_smfmac_applicable(X, ldx, d))) return VNM_ERR_UNSUPPORTED;
  return kProceed;
}

int vnm::spmm_impl(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                     const void* colidx, const void* packed, int64_t out, int64_t in, int V, int N, int M,
                     const Fused& f, void* Y, int64_t ldy, int y_dtype, int path, void* workspace,
                     int64_t workspace_bytes, void* stream) {
  int rc = spmm_validate(X, T, ldx, values, meta, colidx, packed, out, in, V, N, M, f, Y, ldy, y_dtype, path, workspace_bytes);
  if (rc != kProceed) return rc;
  Dims d = make_dims(out, in, V, M);
  hipStream_t st = (hipStream_t)stream;
  const bool fast_ok = packed && has_packed(V, M) && spmm_smfmac_applicable(X, ldx, d);
  if (path == VNM_PATH_SMFMAC && !fast_ok) return VNM_ERR_UNSUPPORTED;
  const int64_t sb = (staged_bytes(T, d) + 255) / 256 * 256;
  const bool xrow_fits = in * 2 <= permute_rows_max_bytes();          // a row of X fits the permuting pass
  if (path != VNM_PATH_GENERIC && fast_ok && T <= skinny_max_tokens() && (!f.perm_in || xrow_fits)) {
    // no staging; a workspace, if given, serves as split-K scratch (same offset as for larger T)
    const bool have = workspace && ((uintptr_t)workspace & 255) == 0 && workspace_bytes > sb;
    const void* Xk = X;
    int64_t ldk = ldx;
    if (f.perm_in) {
      // the kernel reads a permuted copy of X made at the start of the workspace (the region the
      // staged activations occupy for larger T, always large enough for 32 rows of X)
      if (!workspace || workspace_bytes < staged_bytes(T, d)) return VNM_ERR_WORKSPACE;
      if ((uintptr_t)workspace & 255) return VNM_ERR_ALIGN;
      rc = launch_permute_rows(X, ldx, workspace, in, T, in, 2, false, f.perm_in, st);   // in % 8 == 0 here
      if (rc) return rc;
      Xk = workspace; ldk = in;
    }
    return launch_spmm_skinny(Xk, T, ldk, packed, d, Y, ldy, y_dtype, have ? (char*)workspace + sb : nullptr,
                              have ? workspace_bytes - sb : 0, f, st);
  }
  if (path != VNM_PATH_GENERIC && fast_ok) {
    // the matrix-core kernel streams a re-laid copy of X that lives in the caller's workspace
    if (!workspace || workspace_bytes < staged_bytes(T, d)) return VNM_ERR_WORKSPACE;
    if ((uintptr_t)workspace & 255) return VNM_ERR_ALIGN;
    // whatever follows the staged activations serves as split-K scratch, except that with an input
    // permutation and enough room the tail holds a permuted copy of X (made row by row through
    // LDS, which keeps every global access contiguous); without the room, or for rows too long for
    // LDS, the staging pass gathers the permuted columns itself with 2-byte loads (slower).
    int64_t scratch_bytes = workspace_bytes > sb ? workspace_bytes - sb : 0;
    const void* Xk = X;
    int64_t ldk = ldx;
    const int* stage_perm = f.perm_in;
    if (f.perm_in && xrow_fits) {
      const int64_t xp_off = sb + splitk_scratch_bytes(T, out);
      if (workspace_bytes >= xp_off + T * in * 2) {
        rc = launch_permute_rows(X, ldx, (char*)workspace + xp_off, in, T, in, 2, false, f.perm_in, st);
        if (rc) return rc;
        Xk = (char*)workspace + xp_off; ldk = in; stage_perm = nullptr;
        scratch_bytes = xp_off - sb;
      }
    }
    void* scratch = scratch_bytes > 0 ? (char*)workspace + sb : nullptr;
    // a K range that fits LDS (or streams through it for few output channels) needs no staging pass:
    // one kernel straight from X
    // up to 256 tokens where its workgroups fit the compute units at once: the few-token kernel in token groups
    if (!stage_perm && skinny_groups_applicable(T, d, scratch_bytes))
      return launch_spmm_skinny(Xk, T, ldk, packed, d, Y, ldy, y_dtype, scratch, scratch_bytes, f, st);
    if (!stage_perm && spmm_resident_applicable(T, d))
      return launch_spmm_resident(Xk, T, ldk, packed, d, Y, ldy, y_dtype, f, st);
    rc = launch_stage_x(Xk, T, ldk, d, stage_perm, workspace, st);
    if (rc) return rc;
    return launch_spmm_smfmac(workspace, T, packed, d, Y, ldy, y_dtype, scratch, scratch_bytes, f, st);
  }
  return launch_spmm_generic(X, T, ldx, values, meta, colidx, d, Y, ldy, y_dtype, f, st);
}

extern "C" int vnm_spmm(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                        const void* colidx, const void* packed, int64_t out, int64_t in, int V,
                        int N, int M, void* Y, int64_t ldy, int y_dtype, int path, void* workspace,
                        int64_t workspace_bytes, void* stream) {
  return spmm_impl(X, T, ldx, values, meta, colidx, packed, out, in, V, N, M, Fused{}, Y, ldy, y_dtype, path,
                   workspace, workspace_bytes, stream);
}

extern "C" int vnm_spmm_fused(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                              const void* colidx, const void* packed, int64_t out, int64_t in, int V,
                              int N, int M, const void* bias, const void* perm_in, const void* perm_out,
                              void* Y, int64_t ldy, int y_dtype, int path, void* workspace,
                              int64_t workspace_bytes, void* stream) {
  Fused f;
  f.bias = (const _Float16*)bias; f.perm_in = (const int*)perm_in; f.perm_out = (const int*)perm_out;
  if (in > 0x7FFFFFFF || out > 0x7FFFFFFF) return VNM_ERR_UNSUPPORTED;   // 32-bit permutation entries
  return spmm_impl(X, T, ldx, values, meta, colidx, packed, out, in, V, N, M, f, Y, ldy, y_dtype, path,
                   workspace, workspace_bytes, stream);
}

extern "C" int vnm_fold_permutations(const void* perm_out_prev, const void* perm_in_next, int64_t n,
                                     void* folded) {
  if (!perm_out_prev || !perm_in_next || !folded) return VNM_ERR_NULL;
  if (n <= 0 || n > 0x7FFFFFFF) return VNM_ERR_SHAPE;
  const int* po = (const int*)perm_out_prev;
  const int* pi = (const int*)perm_in_next;
  int* res = (int*)folded;
  // both inputs must be permutations of 0..n-1
  try {
  std::vector<int> inv((size_t)n, -1);
  for (int64_t o = 0; o < n; ++o) {
    if (po[o] < 0 || po[o] >= n || inv[(size_t)po[o]] >= 0) return VNM_ERR_SHAPE;
    inv[(size_t)po[o]] = (int)o;
  }
  std::vector<char> seen((size_t)n, 0);
  for (int64_t i = 0; i < n; ++i) {
    if (pi[i] < 0 || pi[i] >= n || seen[(size_t)pi[i]]) return VNM_ERR_SHAPE;
    seen[(size_t)pi[i]] = 1;
  }
  for (int64_t i = 0; i < n; ++i) res[i] = inv[(size_t)pi[i]];
  } catch (...) { return VNM_ERR_WORKSPACE; }                              // out of host memory
  return VNM_OK;
}

extern "C" int vnm_stage_x(const void* X, int64_t T, int64_t ldx, int64_t in, int M, void* staged,
                           int64_t staged_bytes_given, void* stream) {
  if (T != 0 && (!X || !staged)) return VNM_ERR_NULL;
  if (in <= 0 || T < 0 || ldx < in) return VNM_ERR_SHAPE;
  if (M < 4 || M > 16) return VNM_ERR_UNSUPPORTED;
  if (T == 0) return VNM_OK;
  const Dims d = make_dims(64, in, 64, M);                      // the staged layout depends on in and M only
  if (!spmm_smfmac_applicable(X, ldx, d)) return VNM_ERR_UNSUPPORTED;
  if (staged_bytes_given < staged_bytes(T, d)) return VNM_ERR_WORKSPACE;
  if ((uintptr_t)staged & 255) return VNM_ERR_ALIGN;
  return launch_stage_x(X, T, ldx, d, nullptr, staged, (hipStream_t)stream);
}

extern "C" int vnm_spmm_staged(const void* staged, int64_t staged_bytes_given, int64_t T, const void* packed, int64_t out,
                               int64_t in, int V, int N, int M, void* Y, int64_t ldy, int y_dtype,
                               void* scratch, int64_t scratch_bytes, void* stream) {
  if (T != 0 && (!staged || !packed || !Y)) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (T < 0 || ldy < out) return VNM_ERR_SHAPE;
  if (y_dtype != 0 && y_dtype != 1) return VNM_ERR_UNSUPPORTED;
  if (!has_packed(V, M) || in % 8 != 0) return VNM_ERR_UNSUPPORTED;
  if (((uintptr_t)staged & 255) || ((uintptr_t)packed & 255)) return VNM_ERR_ALIGN;
  if ((uintptr_t)Y & (y_dtype == 0 ? 1 : 3)) return VNM_ERR_ALIGN;
  if (scratch_bytes < 0) return VNM_ERR_WORKSPACE;
  if (scratch && ((uintptr_t)scratch & 255)) return VNM_ERR_ALIGN;
  if (T == 0) return VNM_OK;
  // the look-ahead copies of the product kernel read up to three images past the last tile
  if (staged_bytes_given < staged_bytes(T, make_dims(out, in, V, M))) return VNM_ERR_WORKSPACE;
  return launch_spmm_smfmac(staged, T, packed, make_dims(out, in, V, M), Y, ldy, y_dtype, scratch,
                            scratch ? scratch_bytes : 0, Fused{}, (hipStream_t)stream);
}

extern "C" int vnm_spmm_kernel_choice(int64_t T, int64_t out, int64_t in, int V, int N, int M,
                                      int64_t workspace_bytes, int* choice) {
  if (!choice) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (T < 0 || workspace_bytes < 0) return VNM_ERR_SHAPE;
  const Dims d = make_dims(out, in, V, M);
  *choice = VNM_KERNEL_GENERIC;
  if (!has_packed(V, M) || in % 8 != 0) return VNM_OK;
  // (with the workspace vnm_spmm_workspace_bytes asks for)
  if (T <= skinny_max_tokens() || skinny_groups_applicable(T, d, splitk_scratch_bytes(T, out))) { *choice = VNM_KERNEL_FEW_TOKENS; return VNM_OK; }
  *choice = spmm_resident_applicable(T, d) ? VNM_KERNEL_RESIDENT : VNM_KERNEL_STAGED;
  return VNM_OK;
}

extern "C" int vnm_spmm_workspace_bytes(int64_t T, int64_t out, int64_t in, int V, int N, int M,
                                       int64_t* bytes) {
  if (!bytes) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (T < 0) return VNM_ERR_SHAPE;
  *bytes = has_packed(V, M) ? (staged_bytes(T, make_dims(out, in, V, M)) + 255) / 256 * 256 + splitk_scratch_bytes(T, out) : 0;
  return VNM_OK;
}

extern "C" int vnm_spmm_fused_workspace_bytes(int64_t T, int64_t out, int64_t in, int V, int N, int M,
                                             int with_perm_in, int64_t* bytes) {
  int rc = vnm_spmm_workspace_bytes(T, out, in, V, N, M, bytes);
  if (rc) return rc;
  if (with_perm_in && *bytes > 0 && in * 2 <= permute_rows_max_bytes()) *bytes += (T * in * 2 + 255) / 256 * 256;
  return VNM_OK;
}

extern "C" int vnm_stage_x_bytes(int64_t T, int64_t in, int M, int64_t* bytes) {
  if (!bytes) return VNM_ERR_NULL;
  if (in <= 0 || T < 0) return VNM_ERR_SHAPE;
  if (M < 4 || M > 16) return VNM_ERR_UNSUPPORTED;
  *bytes = staged_bytes(T, make_dims(64, in, 64, M));
  return VNM_OK;
}

extern "C" int vnm_spmm_scratch_bytes(int64_t T, int64_t out, int64_t* bytes) {
  if (!bytes) return VNM_ERR_NULL;
  if (out <= 0 || T < 0) return VNM_ERR_SHAPE;
  *bytes = splitk_scratch_bytes(T, out);
  return VNM_OK;
}

extern "C" int vnm_decompress(const void* values, const void* meta, const void* colidx, int64_t out,
                              int64_t in, int V, int N, int M, void* W_out, int64_t ldw,
                              void* stream) {
  if (!values || !meta || !colidx || !W_out) return VNM_ERR_NULL;
  int rc = check_pattern(out, in, V, N, M);
  if (rc) return rc;
  if (ldw < in) return VNM_ERR_SHAPE;
  if (((uintptr_t)W_out & 1) || ((uintptr_t)values & 3)) return VNM_ERR_ALIGN;
  const Dims d = make_dims(out, in, V, M);
  if (decompress_fast_applicable(W_out, ldw, d) && ((uintptr_t)colidx & 3) == 0)
    return launch_decompress_fast(values, meta, colidx, d, W_out, ldw, (hipStream_t)stream);
  return launch_decompress(values, meta, colidx, d, W_out, ldw, (hipStream_t)stream);
}

extern "C" const char* vnm_status_string(int status) {
  switch (status) {
    case VNM_OK: return "ok";
    case VNM_ERR_NULL: return "null pointer";
    case VNM_ERR_SHAPE: return "bad shape or leading dimension";
    case VNM_ERR_UNSUPPORTED: return "unsupported V:N:M, dtype or path";
    case VNM_ERR_ALIGN: return "misaligned pointer";
    case VNM_ERR_WORKSPACE: return "workspace too small";
    case VNM_ERR_HIP: return "HIP error";
    default: return "unknown status";
  }
}

extern "C" const char* vnm_last_hip_error(void) { return vnm::g_hip_error; }
extern "C" int vnm_format_version(void) { return VNM_FORMAT_VERSION; }
