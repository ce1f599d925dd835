// vector_route for callers that cannot allocate: the routing kernels' scratch lives in a
// file-scope device array instead of a caller-provided workspace.
#include <mutex>

#include "../../include/vector.h"
#include "launch.hpp"

namespace {

constexpr size_t kStaticScratchBytes = VECTOR_ROUTE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// One copy per GPU the library runs on, at that GPU's own address; held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress: the device address it stands
// for is looked up once per device below and used everywhere else.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, null until looked up

int scratch_on_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VECTOR_ERR_HIP;
  std::lock_guard<std::mutex> guard(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return VECTOR_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return VECTOR_OK;
}

}  // namespace

extern "C" {

size_t vector_route_static_scratch_bytes(void) { return kStaticScratchBytes; }

int vector_route_static(int32_t n_kv_heads, int32_t seq_len, const float* score, const float* eps, int32_t n_pool,
                        int32_t n_approx, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* stream) {
  if (n_kv_heads < 1 || n_kv_heads > 65535 || seq_len < 1 || seq_len > vec::kRouteMaxSeqLen) return VECTOR_ERR_SHAPE;
  if (n_approx < 0 || n_pool < n_approx || n_pool > seq_len) return VECTOR_ERR_ARG;
  if (!score || !eps || !tier) return VECTOR_ERR_ARG;
  if ((n_pool - n_approx > 0 && !idx_retain) || (n_approx > 0 && !idx_approx)) return VECTOR_ERR_ARG;
  // the same scratch the workspace variant asks its caller for; beyond the array's size: refuse
  if (vec::route_workspace_bytes(n_kv_heads, seq_len, n_pool) > kStaticScratchBytes) return VECTOR_ERR_WORKSPACE;
  void* ptr = nullptr;
  int rc = scratch_on_current_device(&ptr);
  if (rc) return rc;
  return vec::launch_route(n_kv_heads, seq_len, score, eps, n_pool, n_approx, tier, idx_retain, idx_approx, ptr, false,
                           (hipStream_t)stream);
}

}  // extern "C"
