// Asynchronous host <-> device movement of chunk state (declared in chunkft_stream.h):
// hipMemcpyAsync on two copy streams of its own (one per direction), ordered against the
// caller's compute stream and against each other by events.  Default stream priority; no host registration (the caller allocates pinned
// memory itself).

#include <hip/hip_runtime.h>

#include <new>

#include "chunkft.h"
#include "chunkft_stream.h"

// One stream per direction, so that the load of the next chunk and the offload of the previous
// one use both directions of the host link at once.
struct chunkft_mover {
  hipStream_t up = nullptr;        // host -> device
  hipStream_t down = nullptr;      // device -> host
  hipEvent_t fence = nullptr;      // "the compute stream got this far"
  hipEvent_t loaded = nullptr;     // "the most recent load has arrived"
  hipEvent_t offloaded = nullptr;  // "the most recent offload has left the device arrays"
  bool have_load = false, have_offload = false;
};

namespace {
int copy3(hipStream_t on, float* const dst[3], const float* const src[3], int64_t n, hipMemcpyKind kind) {
  const size_t bytes = static_cast<size_t>(n) * sizeof(float);
  for (int i = 0; i < 3; ++i)
    if (hipMemcpyAsync(dst[i], src[i], bytes, kind, on) != hipSuccess) return CHUNKFT_ERR_HIP;
  return CHUNKFT_OK;
}
int order_after(chunkft_mover* mv, hipStream_t copy, void* stream) {
  if (hipEventRecord(mv->fence, static_cast<hipStream_t>(stream)) != hipSuccess) return CHUNKFT_ERR_HIP;
  if (hipStreamWaitEvent(copy, mv->fence, 0) != hipSuccess) return CHUNKFT_ERR_HIP;
  return CHUNKFT_OK;
}
}  // namespace

extern "C" int chunkft_mover_create(chunkft_mover** out) {
  if (!out) return CHUNKFT_ERR_INVALID_ARG;
  *out = nullptr;
  chunkft_mover* mv = new (std::nothrow) chunkft_mover();
  if (!mv) return CHUNKFT_ERR_HIP;
  if (hipStreamCreateWithFlags(&mv->up, hipStreamNonBlocking) != hipSuccess ||
      hipStreamCreateWithFlags(&mv->down, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&mv->fence, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&mv->loaded, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&mv->offloaded, hipEventDisableTiming) != hipSuccess) {
    chunkft_mover_destroy(mv);
    return CHUNKFT_ERR_HIP;
  }
  *out = mv;
  return CHUNKFT_OK;
}

extern "C" void chunkft_mover_destroy(chunkft_mover* mv) {
  if (!mv) return;
  for (hipStream_t st : {mv->up, mv->down})
    if (st) {
      (void)hipStreamSynchronize(st);      // clean-up: nothing to report to
      (void)hipStreamDestroy(st);
    }
  if (mv->fence) (void)hipEventDestroy(mv->fence);
  if (mv->loaded) (void)hipEventDestroy(mv->loaded);
  if (mv->offloaded) (void)hipEventDestroy(mv->offloaded);
  delete mv;
}

extern "C" int chunkft_mover_load(chunkft_mover* mv, float* d_master, float* d_m, float* d_v,
                                  const float* h_master, const float* h_m, const float* h_v, int64_t n,
                                  void* after_stream) {
  if (!mv || !d_master || !d_m || !d_v || !h_master || !h_m || !h_v || n <= 0) return CHUNKFT_ERR_INVALID_ARG;
  int r = order_after(mv, mv->up, after_stream);
  if (r != CHUNKFT_OK) return r;
  // the arrays may still be on their way out
  if (mv->have_offload && hipStreamWaitEvent(mv->up, mv->offloaded, 0) != hipSuccess) return CHUNKFT_ERR_HIP;
  float* const dst[3] = {d_master, d_m, d_v};
  const float* const src[3] = {h_master, h_m, h_v};
  r = copy3(mv->up, dst, src, n, hipMemcpyHostToDevice);
  if (r != CHUNKFT_OK) return r;
  if (hipEventRecord(mv->loaded, mv->up) != hipSuccess) return CHUNKFT_ERR_HIP;
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
  int r = order_after(mv, mv->down, compute_stream);
  if (r != CHUNKFT_OK) return r;
  float* const dst[3] = {h_master, h_m, h_v};
  const float* const src[3] = {d_master, d_m, d_v};
  r = copy3(mv->down, dst, src, n, hipMemcpyDeviceToHost);
  if (r != CHUNKFT_OK) return r;
  if (hipEventRecord(mv->offloaded, mv->down) != hipSuccess) return CHUNKFT_ERR_HIP;
  mv->have_offload = true;
  return CHUNKFT_OK;
}

extern "C" int chunkft_mover_sync(chunkft_mover* mv) {
  if (!mv) return CHUNKFT_ERR_INVALID_ARG;
  if (hipStreamSynchronize(mv->up) != hipSuccess) return CHUNKFT_ERR_HIP;
  return hipStreamSynchronize(mv->down) == hipSuccess ? CHUNKFT_OK : CHUNKFT_ERR_HIP;
}
