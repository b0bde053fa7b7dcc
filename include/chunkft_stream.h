/* Asynchronous movement of a chunk's fp32 state between pinned host memory and the device.
 *
 * Paper: Algorithm 1 -- when a chunk becomes active its master weights and AdamW moments
 * are loaded asynchronously from CPU to GPU, after its last step of the visit they are
 * offloaded asynchronously and the GPU buffers are released; Section 3 (the "streaming"
 * of the active working set).  The chunk-local arrays are the ones the update entry points
 * of chunkft.h work on.  On a 288 GB device a chunk's state need not leave the GPU at all;
 * this is the mechanism for callers that keep it in host memory as the paper does.
 *
 * A mover owns two copy streams (one per direction of the host link) and a few events, no
 * device or host memory.  All copies are
 * ordered by events, never by blocking the host, so the loads of the next chunk and the
 * offload of the previous one run beside the kernels of the active one.  Calls on one mover
 * must come from one thread at a time.
 */
#ifndef CHUNKFT_STREAM_H
#define CHUNKFT_STREAM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct chunkft_mover chunkft_mover;

/* Creates a mover on the current device.  Errors: INVALID_ARG, HIP. */
int chunkft_mover_create(chunkft_mover** out);

/* Waits for the mover's copies, then releases its stream and events.  NULL is allowed. */
void chunkft_mover_destroy(chunkft_mover* mv);

/* Host -> device.  Copies n floats of each of master, m, v from host arrays (pinned, or the
 * copies are not asynchronous) to device arrays.  The copies start only after the work
 * enqueued so far on `after_stream` (kernels that may still use the destination arrays) and
 * after the most recent offload of this mover (which may be out of the same arrays).
 * Returns at once.
 * Errors: INVALID_ARG (null pointer, n <= 0), HIP. */
int chunkft_mover_load(chunkft_mover* mv, float* d_master, float* d_m, float* d_v,
                       const float* h_master, const float* h_m, const float* h_v, int64_t n,
                       void* after_stream);

/* Makes `compute_stream` wait, on the device, until the most recent load has arrived. */
int chunkft_mover_await_load(chunkft_mover* mv, void* compute_stream);

/* Device -> host.  Copies n floats of each array back, after the work enqueued so far on
 * `compute_stream` (the chunk's last update).  Returns at once; the host arrays are valid
 * after chunkft_mover_sync. */
int chunkft_mover_offload(chunkft_mover* mv, float* h_master, float* h_m, float* h_v,
                          const float* d_master, const float* d_m, const float* d_v, int64_t n,
                          void* compute_stream);

/* Blocks the host until every copy enqueued on this mover has finished. */
int chunkft_mover_sync(chunkft_mover* mv);

#ifdef __cplusplus
}
#endif
#endif
