/* Measurement aid of libchunkft: what the matrix cores of the device in use sustain.
 *
 * Not a step of the ChunkFT path.  The published dense bf16 rate of the part
 * assumes its top clock; under a power cap the sustained clock, and with it the
 * rate a contraction can reach, depends on how many operand bits change from one
 * MFMA to the next.  The benchmark reports this measured ceiling beside the
 * fraction of the published peak, so that a reader can tell kernel inefficiency
 * from clock throttling.
 */
#ifndef CHUNKFT_CALIB_H
#define CHUNKFT_CALIB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Device scratch the two calls need: at least this many bytes, 16-byte aligned, owned by
 * the caller like every other buffer of the library (which allocates no device memory). */
#define CHUNKFT_CALIB_SCRATCH_BYTES 4096

/* Runs, on the current device, a kernel that issues nothing but 32x32x16 bf16
 * MFMAs from registers (two waves per SIMD on every compute unit, eight
 * independent accumulator blocks per wave as in the weight-gradient kernel) and
 * times it with HIP events on `stream`.
 *   random_operands  0: all operands are the constant 1.0 (few bits toggle);
 *                    1: operands are random bf16 patterns with exponents around
 *                       one, and every MFMA gets other registers than the one
 *                       before it (the situation of a real contraction).
 *   steps            MFMA steps of 8 instructions per wave; a multiple of 4, >= 4.
 *   scratch          (device) CHUNKFT_CALIB_SCRATCH_BYTES or more; contents are ignored
 *                    on entry and unspecified on return.
 *   tflops           out (host): sustained rate, 2*32*32*16 flop per MFMA.
 *   shader_mhz       out (host): clock during the kernel (shader cycle counter
 *                    against the constant 100 MHz counter).
 * Blocks until the measurement is done (it creates two HIP events for the timing and
 * destroys them before return; no memory is allocated).  Returns CHUNKFT_OK or a
 * negative status: CHUNKFT_ERR_WORKSPACE for a missing, short or misaligned
 * scratch. */
int chunkft_calib_mfma_bf16(int32_t random_operands, int32_t steps, void* scratch, size_t scratch_bytes,
                            double* tflops, double* shader_mhz, void* stream);

/* The same measurement for either bf16 MFMA shape.
 *   shape  32: 32x32x16 (what the call above runs, and what the weight-gradient kernel
 *              issues on its 128 x 256 tile); 16: 16x16x32 (what it issues on its 256 x 256
 *              tile), sixteen per step on 4 x 4 accumulator blocks, the same flop count per
 *              step.  Anything else: CHUNKFT_ERR_INVALID_ARG.
 * The two shapes do the same work per cycle but do not draw the same power, so under
 * the clock limit their sustained rates differ. */
int chunkft_calib_mfma_bf16_shape(int32_t shape, int32_t random_operands, int32_t steps, void* scratch,
                                  size_t scratch_bytes, double* tflops, double* shader_mhz, void* stream);

#ifdef __cplusplus
}
#endif
#endif
