// la_spec_accept for callers that cannot allocate device memory: the kernels of la_spec_accept run on a scratch
// buffer that lives in the library's own image (one copy per GPU the library runs on, held until the process ends)
// instead of a caller-provided workspace.
#include <atomic>
#include <mutex>

#include "la_internal.hpp"

namespace la {
namespace {

// Device array: in host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[LA_SPEC_ACCEPT_STATIC_MAX_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once looked up
std::mutex g_scratch_mutex;

// Address of this device's copy of the array.  Looked up once per device, with that device current.
hipError_t scratch_address(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ptr = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!ptr) {
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!ptr) return hipErrorInvalidSymbol;
      g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
  }
  *out = ptr;
  return hipSuccess;
}

}  // namespace
}  // namespace la

using namespace la;

extern "C" la_status la_spec_accept_static(const la_accept_desc *desc, const void *target_logits,
                                           const void *draft_logits, const int32_t *draft_tokens,
                                           const float *u_accept, const float *u_sample, int32_t *accepted_len,
                                           int32_t *next_token, float *accept_ratio, void *hip_stream) {
  size_t need = 0;
  la_status st = la_spec_accept_workspace(desc, &need);  // validates the descriptor
  if (st != LA_OK) return st;
  if (need > (size_t)LA_SPEC_ACCEPT_STATIC_MAX_BYTES) return LA_ERR_WORKSPACE_TOO_SMALL;
  void *ptr = nullptr;
  if (scratch_address(&ptr) != hipSuccess) return LA_ERR_LAUNCH;
  // every kernel of the path writes what a later one reads of the scratch before it is read, so nothing has to be
  // cleared between calls; what an earlier (larger) call left behind is never looked at
  return la_spec_accept(desc, target_logits, draft_logits, draft_tokens, u_accept, u_sample, accepted_len, next_token,
                        accept_ratio, ptr, (size_t)LA_SPEC_ACCEPT_STATIC_MAX_BYTES, hip_stream);
}
