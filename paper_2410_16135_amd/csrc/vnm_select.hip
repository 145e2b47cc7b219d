// V and M selection (Section 4.1): host-side arithmetic only, no device work.
//
// Among the (V, M) candidates whose measured speedup reaches the threshold, keep for every V the
// smallest M (less sparsity, higher accuracy), then take the candidate of largest mask diversity.
// For a whole network the order of the mask diversities is that of
//     K(V, M) = [C(M,4) * C(4,N)^V]^(1 / (V M))                                   (Eq. 5, Appendix B)
// whatever the layer shapes, so ln K is all that has to be compared.
#include <cmath>
#include "vnm_internal.h"

namespace vnm {

static double ln_k(int V, int M) {
  const double c4 = (double)M * (M - 1) * (M - 2) * (M - 3) / 24.0;      // C(M,4), exact for M <= 255
  return (std::log(c4) + (double)V * std::log(6.0)) / ((double)V * (double)M);
}

}  // namespace vnm

extern "C" int vnm_mask_diversity_log(int V, int N, int M, double* ln_k_out) {
  if (!ln_k_out) return VNM_ERR_NULL;
  if (N != 2 || V < 1 || M < 4 || M > 255) return VNM_ERR_UNSUPPORTED;
  *ln_k_out = vnm::ln_k(V, M);
  return VNM_OK;
}

extern "C" int vnm_select_vm(const int* V, const int* M, const double* speedup, int n, double threshold,
                             int* selected) {
  if (!selected || (n > 0 && (!V || !M || !speedup))) return VNM_ERR_NULL;
  if (n < 0) return VNM_ERR_SHAPE;
  for (int i = 0; i < n; ++i)
    if (V[i] < 1 || M[i] < 4 || M[i] > 255) return VNM_ERR_UNSUPPORTED;
  int best = -1;
  double best_k = 0.0;
  for (int i = 0; i < n; ++i) {
    if (!(speedup[i] >= threshold)) continue;
    // first sifting: i survives only if no qualifying candidate of the same V has a smaller M
    // (of equal (V, M) entries the first one stands for all)
    bool smallest = true;
    for (int j = 0; j < n && smallest; ++j)
      if (j != i && V[j] == V[i] && speedup[j] >= threshold && (M[j] < M[i] || (M[j] == M[i] && j < i)))
        smallest = false;
    if (!smallest) continue;
    // second sifting: largest K; ties to the higher speedup, then to the smaller V, then to the
    // earlier entry
    const double k = vnm::ln_k(V[i], M[i]);
    bool better = best < 0 || k > best_k;
    if (!better && k == best_k) {
      if (speedup[i] > speedup[best]) better = true;
      else if (speedup[i] == speedup[best] && V[i] < V[best]) better = true;
    }
    if (better) { best = i; best_k = k; }
  }
  *selected = best;
  return VNM_OK;
}
