// conv_backward_filter_static: the filter gradient for callers that cannot provide (or allocate) a
// workspace.  The split partials live in a fixed device array that is part of the library's code
// object; the pass itself is the one behind conv_backward_filter, with that array as its workspace.
#include <hip/hip_runtime.h>

#include <mutex>

#include "internal.h"

namespace {

constexpr size_t kScratchBytes = (size_t)32 << 20;  // conv_desc_create keeps the split partials within this
constexpr int kMaxDevices = 64;

// Device memory beyond the caller's blobs: [S][num_output][c/group][kernel_h][kernel_w] partial filter
// gradients.  Every GPU the library runs on holds its own copy at its own address until the process
// ends.  In host code the name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) float scratch[kScratchBytes / sizeof(float)];

std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, looked up once per device
bool g_scratch_known[kMaxDevices];

// The address of this device's copy of `scratch` (the current device), or a HIP error.
int scratch_on_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_known[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!ptr) return (int)hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
    g_scratch_known[dev] = true;
  }
  *out = g_scratch_ptr[dev];
  return 0;
}

}  // namespace

extern "C" int conv_backward_filter_static(const conv_desc_t* d, const float* x, const float* dy, float* dw,
                                           float beta, void* hip_stream) {
  using namespace mi355conv;
  if (!d || !dw) return CONV_EINVAL;
  if (!(beta == 0.f || beta == 1.f)) return CONV_EINVAL;
  if (d->p.n != 0 && (!x || !dy)) return CONV_EINVAL;  // argument errors before any runtime call
  size_t need = 0;
  if (conv_desc_backward_filter_workspace_bytes(d, &need) != CONV_OK) return CONV_EINVAL;
  if (need > kScratchBytes) return CONV_EWORKSPACE;  // this layer's partials do not fit the fixed array
  void* ptr = nullptr;
  if (const int e = scratch_on_current_device(&ptr)) return record_hip_error(e);
  // Nothing in the array has to start at zero: every partial that the reduction reads is written by
  // the filter-gradient kernel of the same call.
  return run_backward_filter(d, x, dy, dw, beta, ptr, kScratchBytes, hip_stream, ReduceExtras());
}

extern "C" size_t conv_static_workspace_limit(void) { return kScratchBytes; }
