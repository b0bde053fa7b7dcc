// Asynchronous host <-> device movement of chunk state (declared in chunkft_stream.h):
// hipMemcpyAsync on a copy stream of its own, ordered against the caller's compute stream
// by events.  Default stream priority; no host registration (the caller allocates pinned
// memory itself).

#include <hip/hip_runtime.h>

#include <new>

#include "chunkft.h"
#include "chunkft_stream.h"

struct chunkft_mover {
  hipStream_t copy = nullptr;
  hipEvent_t fence = nullptr;    // "the compute stream got this far"
  hipEvent_t loaded = nullptr;   // "the most recent load has arrived"
  bool have_load = false;
};

namespace {
int copy3(chunkft_mover* mv, float* const dst[3], const float* const src[3], int64_t n, hipMemcpyKind kind) {
  const size_t bytes = static_cast<size_t>(n) * sizeof(float);
  for (int i = 0; i < 3; ++i)
    if (hipMemcpyAsync(dst[i], src[i], bytes, kind, mv->copy) != hipSuccess) return CHUNKFT_ERR_HIP;
  return CHUNKFT_OK;
}
int order_after(chunkft_mover* mv, void* stream) {
  if (hipEventRecord(mv->fence, static_cast<hipStream_t>(stream)) != hipSuccess) return CHUNKFT_ERR_HIP;
  if (hipStreamWaitEvent(mv->copy, mv->fence, 0) != hipSuccess) return CHUNKFT_ERR_HIP;
  return CHUNKFT_OK;
}
}  // namespace

extern "C" int chunkft_mover_create(chunkft_mover** out) {
  if (!out) return CHUNKFT_ERR_INVALID_ARG;
  *out = nullptr;
  chunkft_mover* mv = new (std::nothrow) chunkft_mover();
  if (!mv) return CHUNKFT_ERR_HIP;
  if (hipStreamCreateWithFlags(&mv->copy, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&mv->fence, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&mv->loaded, hipEventDisableTiming) != hipSuccess) {
    chunkft_mover_destroy(mv);
    return CHUNKFT_ERR_HIP;
  }
  *out = mv;
  return CHUNKFT_OK;
}

extern "C" void chunkft_mover_destroy(chunkft_mover* mv) {
  if (!mv) return;
  if (mv->copy) {
    hipStreamSynchronize(mv->copy);
    hipStreamDestroy(mv->copy);
  }
  if (mv->fence) hipEventDestroy(mv->fence);
  if (mv->loaded) hipEventDestroy(mv->loaded);
  delete mv;
}

extern "C" int chunkft_mover_load(chunkft_mover* mv, float* d_master, float* d_m, float* d_v,
                                  const float* h_master, const float* h_m, const float* h_v, int64_t n,
                                  void* after_stream) {
  if (!mv || !d_master || !d_m || !d_v || !h_master || !h_m || !h_v || n <= 0) return CHUNKFT_ERR_INVALID_ARG;
  int r = order_after(mv, after_stream);
  if (r != CHUNKFT_OK) return r;
  float* const dst[3] = {d_master, d_m, d_v};
  const float* const src[3] = {h_master, h_m, h_v};
  r = copy3(mv, dst, src, n, hipMemcpyHostToDevice);
  if (r != CHUNKFT_OK) return r;
  if (hipEventRecord(mv->loaded, mv->copy) != hipSuccess) return CHUNKFT_ERR_HIP;
  mv->have_load = true;
  return CHUNKFT_OK;
}

extern "C" int chunkft_mover_await_load(chunkft_mover* mv, void* compute_stream) {
  if (!mv) return CHUNKFT_ERR_INVALID_ARG;
  if (!mv->have_load) return CHUNKFT_OK;
  return hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), mv->loaded, 0) == hipSuccess ? CHUNKFT_OK
                                                                                                  : CHUNKFT_ERR_HIP;
}

extern "C" int chunkft_mover_offload(chunkft_mover* mv, float* h_master, float* h_m, float* h_v,
                                     const float* d_master, const float* d_m, const float* d_v, int64_t n,
                                     void* compute_stream) {
  if (!mv || !d_master || !d_m || !d_v || !h_master || !h_m || !h_v || n <= 0) return CHUNKFT_ERR_INVALID_ARG;
  const int r = order_after(mv, compute_stream);
  if (r != CHUNKFT_OK) return r;
  float* const dst[3] = {h_master, h_m, h_v};
  const float* const src[3] = {d_master, d_m, d_v};
  return copy3(mv, dst, src, n, hipMemcpyDeviceToHost);
}

extern "C" int chunkft_mover_sync(chunkft_mover* mv) {
  if (!mv) return CHUNKFT_ERR_INVALID_ARG;
  return hipStreamSynchronize(mv->copy) == hipSuccess ? CHUNKFT_OK : CHUNKFT_ERR_HIP;
}
