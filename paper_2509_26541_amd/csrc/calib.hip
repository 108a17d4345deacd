// Calibration kernels.  Matrix pipe: nothing but matrix instructions, so that a caller who times it
// learns the rate the pipe sustains on this GPU at the clock it actually runs at under load.
// Issue cost: what a vector, a transcendental and an LDS read instruction cost the vector issue port
// of a SIMD next to matrix instructions (the pipe that bounds the attention kernel).
#include <hip/hip_runtime.h>

#include "gfx950.hpp"
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

// Issue-cost calibration.  Every wavefront of a workgroup of eight (two per SIMD, one workgroup
// per CU) repeats a slot of one matrix instruction followed by a few instructions of one kind and
// reports its shader-clock cycles per slot.  The SIMD's arbiter favours the wavefront that was
// launched first, so single wavefronts mislead; the slowest wavefront of a workgroup gives the time
// in which its SIMD issued two slots.  Two wavefronts share a SIMD's vector issue port, so once a
// slot is bound by the port (and not by the 2 x 32 cycles of the matrix pipe) it lasts
// 2 x (matrix instruction + instructions) port cycles: two instruction counts price both terms.
// KIND 0: PER_SLOT v_fma_f32;  1: PER_SLOT v_exp_f32;  2: eight v_fma_f32 and PER_SLOT ds_read_b128
// (1 KiB per wavefront each, waited for a slot later): what the returning LDS data costs the port.
constexpr int ISSUE_BLOCKS = 256, ISSUE_LDS = 96 * 1024;   // the LDS block keeps a second workgroup off the CU

template <int KIND, int PER_SLOT>
__global__ __launch_bounds__(512, 1) void issue_cost_kernel(int64_t* cycles_per_slot_x16, int iters) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[ISSUE_LDS];
  const int tid = threadIdx.x;
  for (int i = tid; i < ISSUE_LDS / 4; i += 512) reinterpret_cast<unsigned*>(lds)[i] = 0x3f803f80u + i;
  __syncthreads();
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  const u32x4 a = {0x3f803f80u + tid, 0x3f813f80u, 0x3f823f80u, 0x3f803f83u};
  const u32x4 b = {0x3f803f80u, 0x3f803f85u + tid, 0x3f863f80u, 0x3f803f87u};
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = 1.0f + 0.125f * i + 1e-3f * tid;
  const float c = 0.75f;
  const unsigned addr = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)lds)) + (tid & 63) * 16 + (tid >> 6) * 8192;
  u32x4 f[2] = {a, a};
  __syncthreads();
  const long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if constexpr (KIND == 2) {
        // the fragments read in the previous slot have landed; one of them feeds the matrix instruction
        asm volatile("s_waitcnt lgkmcnt(0)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(f[0]), "v"(b), "v"(f[1]));
#pragma unroll
        for (int i = 0; i < PER_SLOT; ++i) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[i % 2]) : "v"(addr), "n"(1024 * (i % 8)));
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[i]) : "v"(c));
      } else {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(a), "v"(b));
#pragma unroll
        for (int i = 0; i < PER_SLOT; ++i) {
          if constexpr (KIND == 0) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[(j * PER_SLOT + i) % 8]) : "v"(c));
          else asm volatile("v_exp_f32 %0, %0" : "+v"(x[(j * PER_SLOT + i) % 8]));
        }
      }
    }
  }
  if constexpr (KIND == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]));
  const long long t1 = __builtin_readcyclecounter();
  float r = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[j][i];
#pragma unroll
  for (int i = 0; i < 8; ++i) r += x[i];
  r += __builtin_bit_cast(float, f[0][0]) + __builtin_bit_cast(float, f[1][0]);
  int64_t* mine = cycles_per_slot_x16 + blockIdx.x * 8 + (tid >> 6);
  if ((tid & 63) == 0) *mine = (t1 - t0) * 16 / (static_cast<long long>(iters) * 4);
  if (r == 1.2345e-30f) *mine = 0;      // practically never true; keeps the loop alive
}

template <int KIND, int PER_SLOT>
hipError_t launch_issue_cost(int64_t* out, int iters, hipStream_t stream) {
  return TASP_LAUNCH((issue_cost_kernel<KIND, PER_SLOT>), dim3(ISSUE_BLOCKS), dim3(512), stream, out, iters);
}

}  // namespace
}  // namespace tasp

extern "C" int tasp_calibration_issue(int32_t kind, int32_t per_slot, int32_t iters, int64_t* cycles_per_slot_x16,
                                      void* hip_stream) {
  if (iters < 1 || iters > (1 << 20) || cycles_per_slot_x16 == nullptr) return TASP_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipErrorInvalidValue;
  if (kind == 0 && per_slot == 8) e = tasp::launch_issue_cost<0, 8>(cycles_per_slot_x16, iters, st);
  else if (kind == 0 && per_slot == 12) e = tasp::launch_issue_cost<0, 12>(cycles_per_slot_x16, iters, st);
  else if (kind == 1 && per_slot == 4) e = tasp::launch_issue_cost<1, 4>(cycles_per_slot_x16, iters, st);
  else if (kind == 1 && per_slot == 8) e = tasp::launch_issue_cost<1, 8>(cycles_per_slot_x16, iters, st);
  else if (kind == 2 && per_slot == 1) e = tasp::launch_issue_cost<2, 1>(cycles_per_slot_x16, iters, st);
  else if (kind == 2 && per_slot == 2) e = tasp::launch_issue_cost<2, 2>(cycles_per_slot_x16, iters, st);
  else return TASP_EINVAL;
  return e == hipSuccess ? TASP_OK : TASP_EHIP;
}

extern "C" int tasp_calibration_mfma(int32_t iters, double* flops, void* hip_stream) {
  if (iters < 1 || iters > (1 << 20)) return TASP_EINVAL;
  if (flops != nullptr)
    *flops = static_cast<double>(tasp::CALIB_BLOCKS) * tasp::CALIB_WAVES * iters * tasp::CALIB_MFMA_PER_ITER *
             (2.0 * 32 * 32 * 16);
  const hipError_t e = TASP_LAUNCH(tasp::mfma_peak_kernel, dim3(tasp::CALIB_BLOCKS), dim3(64 * tasp::CALIB_WAVES),
                                   static_cast<hipStream_t>(hip_stream), static_cast<float*>(nullptr), iters);
  return e == hipSuccess ? TASP_OK : TASP_EHIP;
}
