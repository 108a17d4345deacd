// Matrix-pipe calibration: nothing but matrix instructions, so that a caller who times it learns the
// rate the pipe sustains on this GPU at the clock it actually runs at under load.
#include <hip/hip_runtime.h>

#include "internal.hpp"
#include "tasp.h"

namespace tasp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int CALIB_BLOCKS = 2048, CALIB_WAVES = 8, CALIB_MFMA_PER_ITER = 32;

__global__ __launch_bounds__(64 * CALIB_WAVES, 2) void mfma_peak_kernel(float* sink, int iters) {
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  // operands with the statistics of real activations (pseudo-random, zero mean, magnitude about one):
  // the clock the pipe sustains depends on how many bits toggle
  bf16x8 a, b;
  unsigned h = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    h = h * 1664525u + 1013904223u;
    a[i] = static_cast<__bf16>(static_cast<float>(static_cast<int>(h >> 16) - 32768) * (1.0f / 16384.0f));
    h = h * 1664525u + 1013904223u;
    b[i] = static_cast<__bf16>(static_cast<float>(static_cast<int>(h >> 16) - 32768) * (1.0f / 16384.0f));
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < CALIB_MFMA_PER_ITER; ++q)
      acc[q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q & 3], 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[j][i];
  if (r == 1.2345e-30f && sink != nullptr) *sink = r;      // practically never true; keeps the loop alive
}

}  // namespace
}  // namespace tasp

extern "C" int tasp_calibration_mfma(int32_t iters, double* flops, void* hip_stream) {
  if (iters < 1 || iters > (1 << 20)) return TASP_EINVAL;
  if (flops != nullptr)
    *flops = static_cast<double>(tasp::CALIB_BLOCKS) * tasp::CALIB_WAVES * iters * tasp::CALIB_MFMA_PER_ITER *
             (2.0 * 32 * 32 * 16);
  const hipError_t e = TASP_LAUNCH(tasp::mfma_peak_kernel, dim3(tasp::CALIB_BLOCKS), dim3(64 * tasp::CALIB_WAVES),
                                   static_cast<hipStream_t>(hip_stream), static_cast<float*>(nullptr), iters);
  return e == hipSuccess ? TASP_OK : TASP_EHIP;
}
