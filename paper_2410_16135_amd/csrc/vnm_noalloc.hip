// vnm_spmm_noalloc: vnm_spmm with its workspace as a device array inside the library image, for
// callers that cannot allocate or hand over one.  The array and the call that takes its device
// address live in this one file: in host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it yields (one per device, each GPU has its own copy) is
// what kernels and size checks use.
#include <stdio.h>
#include <mutex>
#include <utility>
#include <vector>
#include "vnm_internal.h"

using namespace vnm;

static __device__ __align__(256) unsigned char scratch[VNM_NOALLOC_SCRATCH_BYTES];

static int noalloc_scratch(void** ptr_out) {
  static std::mutex mu;
  static std::vector<std::pair<int, void*>> per_device;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_hip_error(e, "hipGetDevice"); return VNM_ERR_HIP; }
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& p : per_device)
    if (p.first == dev) { *ptr_out = p.second; return VNM_OK; }
  void* ptr = nullptr;
  e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !ptr) { set_hip_error(e, "hipGetSymbolAddress(scratch)"); return VNM_ERR_HIP; }
  per_device.push_back({dev, ptr});
  *ptr_out = ptr;
  return VNM_OK;
}

extern "C" int vnm_spmm_noalloc(const void* X, int64_t T, int64_t ldx, const void* values, const void* meta,
                                const void* colidx, const void* packed, int64_t out, int64_t in, int V, int N,
                                int M, void* Y, int64_t ldy, int y_dtype, int path, void* stream) {
  // argument and size checks first (host arithmetic only): a bad or oversized request never
  // touches the device
  int rc = spmm_validate(X, T, ldx, values, meta, colidx, packed, out, in, V, N, M, Fused{}, Y, ldy, y_dtype, path, 0);
  if (rc != kProceed) return rc;
  if (has_packed(V, M)) {
    const Dims d = make_dims(out, in, V, M);
    const int64_t need = (staged_bytes(T, d) + 255) / 256 * 256;
    const bool staged_path = path != VNM_PATH_GENERIC && packed && spmm_smfmac_applicable(X, ldx, d) &&
                             T > skinny_max_tokens();
    if (staged_path && need > (int64_t)VNM_NOALLOC_SCRATCH_BYTES) {
      char msg[256];
      snprintf(msg, sizeof(msg),
               "vnm_spmm_noalloc: %lld tokens x %lld input channels need %lld bytes of staged activations, the "
               "built-in scratch holds %lld; use vnm_spmm with a workspace",
               (long long)T, (long long)in, (long long)need, (long long)VNM_NOALLOC_SCRATCH_BYTES);
      set_error_text(msg);
      return VNM_ERR_WORKSPACE;
    }
  }
  void* ws = nullptr;
  if ((rc = noalloc_scratch(&ws)) != VNM_OK) return rc;
  return spmm_impl(X, T, ldx, values, meta, colidx, packed, out, in, V, N, M, Fused{}, Y, ldy, y_dtype, path, ws,
                   (int64_t)VNM_NOALLOC_SCRATCH_BYTES, stream);
}

