// The fused call for callers that cannot hand over (or allocate) a workspace: the token-slab
// partial sums and the per-token statistics live in a device array that is part of the library's
// code object, one copy per GPU, held until the process ends.

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "chunkft.h"
#include "internal.h"

namespace {

// Device memory of the code object.  In host code this name is only a handle for
// hipGetSymbolAddress: the address a kernel (or any runtime call) may use is the one that call
// returns for the current device, kept in g_scratch_ptr below.
static __device__ __align__(256) unsigned char scratch[CHUNKFT_STATIC_WORKSPACE_BYTES];

std::atomic<void*> g_scratch_ptr[chunkft::kMaxDevices] = {};

// Address of the current device's copy of the array; asked of the runtime once per device.
int scratch_of_current_device(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= chunkft::kMaxDevices) {
    (void)hipGetLastError();
    return CHUNKFT_ERR_HIP;
  }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return CHUNKFT_ERR_HIP;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing store the same address
  }
  *out = p;
  return CHUNKFT_OK;
}

}  // namespace

extern "C" int chunkft_wgrad_adamw_fused_static(const chunkft_layer* L, int64_t begin, int64_t end, void* W,
                                                float* master, float* m, float* v,
                                                const chunkft_adamw_hparams* hp, void* stream) {
  // 0 for invalid arguments too: the call below then reports them, before it looks at the workspace
  const size_t need = chunkft_workspace_bytes(L, begin, end);
  if (need > (size_t)CHUNKFT_STATIC_WORKSPACE_BYTES) return CHUNKFT_ERR_STATIC_WORKSPACE;
  void* ws = nullptr;
  if (need > 0) {
    const int r = scratch_of_current_device(&ws);
    if (r != CHUNKFT_OK) return r;
  }
  // Nothing in the array has to start at zero: every word the reduction (or the normalising
  // operator) reads is written earlier in the same call, by the slab kernels (or the statistics
  // kernel), so what the previous call left behind is never seen.
  return chunkft_wgrad_adamw_fused(L, begin, end, W, master, m, v, hp, ws, need > 0 ? (size_t)CHUNKFT_STATIC_WORKSPACE_BYTES : 0, stream);
}
