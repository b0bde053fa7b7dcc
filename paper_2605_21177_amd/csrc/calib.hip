// Sustained MFMA rate of the device: the measurement aid declared in chunkft_calib.h.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "chunkft.h"
#include "chunkft_calib.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// A pool of 16 A and 8 B fragments stays in registers; step s of four uses A[4s..4s+3] and
// B[2s], B[2s+1], ... (modulo 8), so consecutive MFMAs of a SIMD never see the same
// operands (when RANDOM).  SHAPE 32: eight 32x32x16 MFMAs per step on 4 x 2 accumulator
// blocks; SHAPE 16: sixteen 16x16x32 MFMAs per step on 4 x 4 blocks -- the same flop
// count, the same operand pool.
template <int SHAPE, int RANDOM>
__global__ __launch_bounds__(256, 2) void mfma_rate_kernel(float* sink, int steps, unsigned long long* clk) {
  u32x4 a[16], b[8];
  unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  auto pattern = [&]() {
    s = s * 1664525u + 1013904223u;
    const unsigned mant = (s >> 9) & 0x007f007fu, sign = s & 0x80008000u, expo = (s >> 3) & 0x03000300u;
    return RANDOM ? ((0x3e003e00u + expo) | mant | sign) : 0x3f803f80u;   // two bf16 per word
  };
  for (int i = 0; i < 16; ++i)
    for (int e = 0; e < 4; ++e) a[i][e] = pattern();
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) b[i][e] = pattern();
  constexpr int NJ = SHAPE == 32 ? 2 : 4, NV = SHAPE == 32 ? 16 : 4;
  using acc_t = typename std::conditional<SHAPE == 32, f32x16, f32x4>::type;
  acc_t acc[4][NJ];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < NJ; ++j)
      for (int v = 0; v < NV; ++v) acc[i][j][v] = 0.f;
  const unsigned long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < steps; it += 4) {
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const bf16x8 fa = __builtin_bit_cast(bf16x8, a[st * 4 + i]);
          const bf16x8 fb = __builtin_bit_cast(bf16x8, b[(st * 2 + j) & 7]);
          if constexpr (SHAPE == 32) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[i][j], 0, 0, 0);
          else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc[i][j], 0, 0, 0);
        }
  }
  const unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float sum = 0;
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < NJ; ++j)
      for (int v = 0; v < NV; ++v) sum += acc[i][j][v];
  if (sum == 12345.678f) sink[threadIdx.x] = sum;      // keeps the accumulators alive; never true in practice
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clk[0] = t1 - t0;
    clk[1] = r1 - r0;
  }
}

}  // namespace

extern "C" int chunkft_calib_mfma_bf16(int32_t random_operands, int32_t steps, void* scratch, size_t scratch_bytes,
                                       double* tflops, double* shader_mhz, void* stream) {
  return chunkft_calib_mfma_bf16_shape(32, random_operands, steps, scratch, scratch_bytes, tflops, shader_mhz, stream);
}

extern "C" int chunkft_calib_mfma_bf16_shape(int32_t shape, int32_t random_operands, int32_t steps, void* scratch,
                                             size_t scratch_bytes, double* tflops, double* shader_mhz, void* stream) {
  if (!tflops || !shader_mhz || steps < 4 || steps % 4 != 0 || steps > (1 << 20)) return CHUNKFT_ERR_INVALID_ARG;
  if (shape != 32 && shape != 16) return CHUNKFT_ERR_INVALID_ARG;
  if (!scratch || scratch_bytes < CHUNKFT_CALIB_SCRATCH_BYTES || (reinterpret_cast<uintptr_t>(scratch) & 15u))
    return CHUNKFT_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return CHUNKFT_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return CHUNKFT_ERR_HIP;
  float* sink = (float*)scratch;
  unsigned long long* clk = (unsigned long long*)((char*)scratch + 2048);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = CHUNKFT_ERR_HIP;
  const int grid = 2 * cus, reps = 5;
  auto launch = [&]() {
    auto k = shape == 32 ? (random_operands ? mfma_rate_kernel<32, 1> : mfma_rate_kernel<32, 0>)
                         : (random_operands ? mfma_rate_kernel<16, 1> : mfma_rate_kernel<16, 0>);
    hipLaunchKernelGGL(k, dim3(grid), dim3(256), 0, st, sink, steps, clk);
  };
  do {
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
    for (int i = 0; i < 2; ++i) launch();
    if (hipEventRecord(e0, st) != hipSuccess) break;
    for (int i = 0; i < reps; ++i) launch();
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) break;
    if (hipGetLastError() != hipSuccess) break;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) break;
    unsigned long long h[2] = {0, 0};
    if (hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess || h[1] == 0) break;
    const double flop = 2.0 * 32 * 32 * 16 * 8.0 * steps * 4.0 * grid * reps;   // per step and wave, either shape
    *tflops = flop / (ms * 1e-3) / 1e12;
    *shader_mhz = (double)h[0] / (double)h[1] * 100.0;
    rc = CHUNKFT_OK;
  } while (false);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  return rc;
}
