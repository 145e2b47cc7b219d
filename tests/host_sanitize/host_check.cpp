// Host-only check of libvnm's host code paths under AddressSanitizer and UndefinedBehaviorSanitizer:
// the assignment solver, the V/M selection, the folding of permutations, the size queries and the
// argument validation of every entry point (everything that runs before a kernel is launched).
// Built by tests/test_host_sanitizers.py from csrc/vnm_api.hip, vnm_lsa.hip and vnm_select.hip with
// the host pass only; the kernel launchers those files call are replaced by the stubs below, which
// fail the run if any of them is reached.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <numeric>
#include <random>
#include <vector>
#include "vnm_internal.h"

static int g_launches = 0;
namespace vnm {
#define STUB { ++g_launches; return 77; }
int launch_lora_merge(const void*, int64_t, const void*, int64_t, const void*, int64_t, int, float, int64_t, int64_t, void*, int64_t, hipStream_t) STUB
int launch_pack(const void*, const void*, const void*, const Dims&, void*, hipStream_t) STUB
int launch_permute_rows(const void*, int64_t, void*, int64_t, int64_t, int64_t, int, bool, const int*, hipStream_t) STUB
int launch_prune_compress(const void*, int64_t, const Dims&, void*, void*, void*, void*, hipStream_t) STUB
int launch_prune_fast(const void*, int64_t, const Dims&, void*, void*, void*, void*, void*, hipStream_t) STUB
int launch_prune_fast_scored(const void*, int64_t, const void*, int64_t, const Dims&, void*, void*, void*, void*, void*, hipStream_t) STUB
int launch_prune_scored(const void*, int64_t, const void*, int64_t, const Dims&, void*, void*, void*, void*, hipStream_t) STUB
int launch_ria_scores(const void*, int64_t, int64_t, int64_t, const void*, void*, int64_t, void*, hipStream_t) STUB
int launch_spmm_generic(const void*, int64_t, int64_t, const void*, const void*, const void*, const Dims&, void*, int64_t, int, const Fused&, hipStream_t) STUB
int launch_spmm_resident(const void*, int64_t, int64_t, const void*, const Dims&, void*, int64_t, int, const Fused&, hipStream_t) STUB
int launch_spmm_skinny(const void*, int64_t, int64_t, const void*, const Dims&, void*, int64_t, int, void*, int64_t, const Fused&, hipStream_t) STUB
int launch_stage_x(const void*, int64_t, int64_t, const Dims&, const int*, void*, hipStream_t) STUB
int launch_spmm_smfmac(const void*, int64_t, const void*, const Dims&, void*, int64_t, int, void*, int64_t, const Fused&, hipStream_t) STUB
int launch_decompress(const void*, const void*, const void*, const Dims&, void*, int64_t, hipStream_t) STUB
int launch_decompress_fast(const void*, const void*, const void*, const Dims&, void*, int64_t, hipStream_t) STUB
#undef STUB
// host helpers that live next to kernels in the library: stand-ins with the same meaning
int64_t permute_rows_max_bytes() { return 144 * 1024; }
int64_t skinny_max_tokens() { return 32; }
int64_t splitk_scratch_bytes(int64_t T, int64_t out) { return T > 0 && T <= 2048 ? std::min<int64_t>(16 * T * out * 4, 64ll << 20) : 0; }
int64_t staged_bytes(int64_t T, const Dims& d) { return ((T + kTokTile - 1) / kTokTile * d.S + 3) * image_bytes(d.M); }
bool prune_fast_applicable(const void*, int64_t, const Dims&, const void*) { return true; }
bool prune_fast_scored_applicable(const void*, int64_t, const void*, int64_t, const Dims&) { return true; }
bool decompress_fast_applicable(const void*, int64_t, const Dims&) { return true; }
bool spmm_resident_applicable(int64_t, const Dims&) { return false; }
bool skinny_groups_applicable(int64_t, const Dims&, int64_t) { return false; }
bool spmm_smfmac_applicable(const void* X, int64_t ldx, const Dims& d) {
  return has_packed(d.V, d.M) && d.in % 8 == 0 && ldx % 8 == 0 && ((uintptr_t)X & 15) == 0;
}
}  // namespace vnm

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "host_check: %s failed at line %d\n", #c, __LINE__); return 1; } } while (0)

static int64_t brute_force(const std::vector<int64_t>& g, int n) {
  std::vector<int> p((size_t)n);
  std::iota(p.begin(), p.end(), 0);
  int64_t best = -1;
  do {
    int64_t s = 0;
    for (int i = 0; i < n; ++i) s += g[(size_t)i * n + p[(size_t)i]];
    best = std::max(best, s);
  } while (std::next_permutation(p.begin(), p.end()));
  return best;
}

int main() {
  std::mt19937_64 rng(7);
  // ---- assignment solver: optimum against enumeration (ties included), validity on larger inputs
  for (int n = 1; n <= 7; ++n)
    for (int rep = 0; rep < 20; ++rep) {
      std::vector<int64_t> g((size_t)n * n);
      for (auto& v : g) v = (int64_t)(rng() % (rep % 2 ? 4 : 1000000));
      std::vector<int> as((size_t)n, -1);
      int64_t tot = -1;
      CHECK(vnm_lsa_max(g.data(), n, as.data(), &tot) == VNM_OK);
      CHECK(tot == brute_force(g, n));
      { std::vector<int> as2((size_t)n, -1); int64_t t2 = -1;
        CHECK(vnm_lsa_max_method(g.data(), n, VNM_LSA_HUNGARIAN, as2.data(), &t2) == VNM_OK && t2 == tot);
        CHECK(vnm_lsa_max_method(g.data(), n, VNM_LSA_AUCTION, as2.data(), &t2) == VNM_OK && t2 == tot);
        CHECK(vnm_lsa_max_method(g.data(), n, VNM_LSA_AUCTION_SCALAR, as2.data(), &t2) == VNM_OK && t2 == tot); }
      std::vector<char> seen((size_t)n, 0);
      int64_t sum = 0;
      for (int i = 0; i < n; ++i) { CHECK(as[(size_t)i] >= 0 && as[(size_t)i] < n && !seen[(size_t)as[(size_t)i]]); seen[(size_t)as[(size_t)i]] = 1; sum += g[(size_t)i * n + as[(size_t)i]]; }
      CHECK(sum == tot);
    }
  for (int n : {33, 200, 511}) {
    std::vector<int64_t> g((size_t)n * n);
    // a few attractive columns and a baseline per column, the shape of the search's gain matrices
    for (int i = 0; i < n; ++i) for (int j = 0; j < n; ++j) g[(size_t)i * n + j] = (int64_t)(1000000 + 1000 * j + (j % 17 == 0 ? rng() % 50000 : rng() % 50));
    std::vector<int> as((size_t)n, -1);
    int64_t tot = -1;
    CHECK(vnm_lsa_max(g.data(), n, as.data(), &tot) == VNM_OK);
    std::vector<char> seen((size_t)n, 0);
    int64_t sum = 0, ident = 0;
    for (int i = 0; i < n; ++i) { CHECK(as[(size_t)i] >= 0 && as[(size_t)i] < n && !seen[(size_t)as[(size_t)i]]); seen[(size_t)as[(size_t)i]] = 1; sum += g[(size_t)i * n + as[(size_t)i]]; ident += g[(size_t)i * n + i]; }
    CHECK(sum == tot && tot >= ident);
    { std::vector<int> as2((size_t)n, -1); int64_t t2 = -1;       // both methods, same optimum
      CHECK(vnm_lsa_max_method(g.data(), n, VNM_LSA_HUNGARIAN, as2.data(), &t2) == VNM_OK && t2 == tot);
      CHECK(vnm_lsa_max_method(g.data(), n, VNM_LSA_AUCTION, as2.data(), &t2) == VNM_OK && t2 == tot);
      CHECK(vnm_lsa_max_method(g.data(), n, VNM_LSA_AUCTION_SCALAR, as2.data(), &t2) == VNM_OK && t2 == tot); }
  }
  { int64_t bad[4] = {1, -1, 2, 3}; int as[2]; int64_t tot; CHECK(vnm_lsa_max(bad, 2, as, &tot) == VNM_ERR_SHAPE); CHECK(vnm_lsa_max(nullptr, 2, as, &tot) == VNM_ERR_NULL); CHECK(vnm_lsa_max(bad, 0, as, &tot) == VNM_ERR_SHAPE); }
  // ---- V/M selection
  { double k5 = 0, k8 = 0; CHECK(vnm_mask_diversity_log(64, 2, 5, &k5) == VNM_OK && vnm_mask_diversity_log(64, 2, 8, &k8) == VNM_OK && k5 > k8 && k8 > 0);
    CHECK(vnm_mask_diversity_log(64, 3, 5, &k5) == VNM_ERR_UNSUPPORTED);
    int V[6] = {32, 32, 64, 64, 128, 128}, M[6] = {5, 8, 5, 8, 6, 16}; double sp[6] = {1.1, 1.6, 1.3, 1.9, 1.5, 3.0}; int sel = -2;
    CHECK(vnm_select_vm(V, M, sp, 6, 1.25, &sel) == VNM_OK && sel >= 0 && sel < 6);
    CHECK(vnm_select_vm(V, M, sp, 6, 9.0, &sel) == VNM_OK && sel == -1);
    CHECK(vnm_select_vm(V, M, sp, 0, 1.0, &sel) == VNM_OK && sel == -1); }
  // ---- folding of permutations
  for (int64_t n : {1, 2, 17, 4096}) {
    std::vector<int> po((size_t)n), pi((size_t)n), folded((size_t)n, -1);
    std::iota(po.begin(), po.end(), 0); std::iota(pi.begin(), pi.end(), 0);
    std::shuffle(po.begin(), po.end(), rng); std::shuffle(pi.begin(), pi.end(), rng);
    CHECK(vnm_fold_permutations(po.data(), pi.data(), n, folded.data()) == VNM_OK);
    for (int64_t i = 0; i < n; ++i) CHECK(po[(size_t)folded[(size_t)i]] == pi[(size_t)i]);
    if (n >= 2) { std::vector<int> dup = po; dup[0] = dup[1]; CHECK(vnm_fold_permutations(dup.data(), pi.data(), n, folded.data()) == VNM_ERR_SHAPE);
                  std::vector<int> oob = pi; oob[(size_t)n - 1] = (int)n; CHECK(vnm_fold_permutations(po.data(), oob.data(), n, folded.data()) == VNM_ERR_SHAPE); }
  }
  CHECK(vnm_fold_permutations(nullptr, nullptr, 4, nullptr) == VNM_ERR_NULL);
  // ---- size queries and argument validation: every call below must return before any launch
  { vnm_sizes s; CHECK(vnm_query_sizes(4096, 11008, 64, 2, 5, &s) == VNM_OK && s.col_blocks == 2202 && s.out_pad == 4096 && s.kc == 8808);
    CHECK(vnm_query_sizes(4096, 11008, 64, 2, 3, &s) == VNM_ERR_UNSUPPORTED && vnm_query_sizes(0, 8, 64, 2, 5, &s) == VNM_ERR_SHAPE);
    int64_t b = -1; CHECK(vnm_spmm_workspace_bytes(4096, 4096, 4096, 64, 2, 5, &b) == VNM_OK && b > 0);
    CHECK(vnm_stage_x_bytes(4096, 4096, 17, &b) == VNM_ERR_UNSUPPORTED && vnm_spmm_scratch_bytes(16, 0, &b) == VNM_ERR_SHAPE);
    int ch = -1; CHECK(vnm_spmm_kernel_choice(16, 4096, 4096, 64, 2, 5, 0, &ch) == VNM_OK && ch == VNM_KERNEL_FEW_TOKENS);
    CHECK(vnm_spmm_kernel_choice(4096, 4096, 4100, 64, 2, 5, 0, &ch) == VNM_OK && ch == VNM_KERNEL_GENERIC); }
  { void* good = (void*)0x1000; void* odd = (void*)0x1001;
    CHECK(vnm_prune_compress(nullptr, 128, 128, 128, 64, 2, 8, good, good, good, nullptr, nullptr, nullptr, 0, nullptr) == VNM_ERR_NULL);
    CHECK(vnm_prune_compress(odd, 128, 128, 128, 64, 2, 8, good, good, good, nullptr, nullptr, nullptr, 0, nullptr) == VNM_ERR_ALIGN);
    CHECK(vnm_spmm(good, 4, 127, good, good, good, nullptr, 128, 128, 64, 2, 8, good, 128, 0, 0, nullptr, 0, nullptr) == VNM_ERR_SHAPE);
    CHECK(vnm_spmm(good, 64, 128, good, good, good, good, 128, 128, 64, 2, 8, good, 128, 0, 0, nullptr, 0, nullptr) == VNM_ERR_WORKSPACE);
    CHECK(vnm_spmm(nullptr, 0, 128, good, good, good, nullptr, 128, 128, 64, 2, 8, nullptr, 128, 0, 0, nullptr, 0, nullptr) == VNM_OK);
    CHECK(vnm_spmm_fused(good, 4, 128, good, good, good, nullptr, 128, 128, 64, 2, 8, odd, nullptr, nullptr, good, 128, 0, 0, nullptr, 0, nullptr) == VNM_ERR_ALIGN);
    CHECK(vnm_spmm_staged(good, 16, 4, good, 128, 128, 64, 2, 8, good, 128, 0, nullptr, 0, nullptr) == VNM_ERR_WORKSPACE);
    CHECK(vnm_decompress(good, good, good, 128, 128, 64, 2, 8, good, 5, nullptr) == VNM_ERR_SHAPE);
    CHECK(vnm_pack(good, good, good, 128, 128, 16, 2, 8, good, nullptr) == VNM_ERR_UNSUPPORTED);
    CHECK(vnm_ria_scores(good, 8, 8, 8, good, good, 8, good, 127, nullptr) == VNM_ERR_WORKSPACE);
    CHECK(vnm_lora_merge(good, 8, 8, 8, nullptr, 4, good, 8, 4, 2.0f, good, 8, nullptr) == VNM_ERR_NULL);
    CHECK(vnm_prune_compress_scored(good, good, 128, 128, 128, 100, 64, 2, 8, good, good, good, nullptr, nullptr, nullptr) == VNM_ERR_SHAPE); }
  CHECK(g_launches == 0);
  printf("host_check ok\n");
  return 0;
}
