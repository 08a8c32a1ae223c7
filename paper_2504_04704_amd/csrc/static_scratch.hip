// lagkv_compress_static: lagkv_compress for callers that cannot allocate (code under HIP
// graph capture, tight serving loops).  The three-kernel path stages its scores and kept
// positions in a fixed device array that this file owns instead of a caller's workspace.
#include <hip/hip_runtime.h>

#include <mutex>

#include "lagkv.h"
#include "lagkv_internal.hpp"

namespace {

constexpr size_t kScratchBytes = LAGKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// One copy per GPU that loads the library, held until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress; kernels receive the resolved address.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_lock;
void* g_scratch_addr[kMaxDevices] = {};

// Device address of `scratch` on the current device (resolved once per device).
int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LAGKV_EHIP;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_addr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LAGKV_EHIP;
    g_scratch_addr[dev] = ptr;
  }
  *out = g_scratch_addr[dev];
  return LAGKV_OK;
}

}  // namespace

extern "C" int lagkv_compress_static(const lagkv_params* p, const void* K, const void* V, int64_t T,
                                     void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                                     void* hip_stream) {
  const size_t need = lagkv::compress_workspace_need(p, T);
  if (need > kScratchBytes) return LAGKV_EWORKSPACE;  // beyond the static scratch: use lagkv_compress
  void* ws = nullptr;
  if (need > 0) {
    const int rc = scratch_of_current_device(&ws);
    if (rc != LAGKV_OK) return rc;
  }
  // every word of the scratch that a kernel reads is written earlier in the same call
  // (scores by the scoring kernel, kept positions by the selection kernel): nothing has to
  // start at zero
  return lagkv::compress_with_workspace(p, K, V, T, K_out, V_out, idx_out, scores_out, ws, need,
                                        hip_stream);
}
