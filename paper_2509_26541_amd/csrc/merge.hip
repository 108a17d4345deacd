// update_out_lse of Algorithm 3 as a streaming kernel, plus the two small helpers around it
// (mark rows that saw no key; cast the fp32 result to bf16).  All three are bound by HBM traffic:
// every thread moves 16-byte pieces, consecutive lanes touch consecutive addresses.
#include <hip/hip_runtime.h>

#include "internal.hpp"
#include "tasp.h"

namespace tasp {
inline namespace merge_detail {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int MERGE_THREADS = 256;

// One thread per 4 output columns of one (row, head).  n4 = rows*heads*d/4, pieces = d/4.  The
// second grid dimension walks the sequences of a batch (the same row range of each): bstride_rh =
// (row, head) pairs from one sequence to the next.
__global__ __launch_bounds__(MERGE_THREADS) void merge_kernel(float* __restrict__ o_acc, float* __restrict__ lse_acc,
                                                             const float* __restrict__ o_part,
                                                             const float* __restrict__ lse_part, int64_t n4,
                                                             int32_t pieces, int64_t bstride_rh) {
  const int64_t boff = static_cast<int64_t>(blockIdx.y) * bstride_rh;
  o_acc += boff * pieces * 4; o_part += boff * pieces * 4; lse_acc += boff; lse_part += boff;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * MERGE_THREADS;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * MERGE_THREADS + threadIdx.x; i < n4; i += stride) {
    const int64_t rh = i / pieces;
    const float la = lse_acc[rh], lb = lse_part[rh];
    const f32x4 a = reinterpret_cast<const f32x4*>(o_acc)[i];
    const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(o_part) + i);
    const float mx = fmaxf(la, lb);
    f32x4 r;
    float lnew;
    if (mx == -__builtin_inff()) {
      r = f32x4{0.f, 0.f, 0.f, 0.f};
      lnew = mx;
    } else {
      const float ea = __expf(la - mx), eb = __expf(lb - mx);
      const float den = ea + eb, rden = 1.f / den;
      const float wa = ea * rden, wb = eb * rden;
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = wa * a[e] + wb * b[e];
      lnew = mx + __logf(den);
    }
    reinterpret_cast<f32x4*>(o_acc)[i] = r;
    // d/4 divides 64, so all pieces of a (row, head) sit in one wavefront: its load of la above
    // was issued for every lane before this store
    if (i - rh * pieces == 0) lse_acc[rh] = lnew;
  }
}

// N partials in one pass.  The pointers travel in the kernel argument block.
struct ManyParts {
  const float* o[TASP_MAX_MERGE_PARTS];
  const float* lse[TASP_MAX_MERGE_PARTS];
};

__global__ __launch_bounds__(MERGE_THREADS) void merge_many_kernel(float* __restrict__ o_out, float* __restrict__ lse_out,
                                                                  const ManyParts parts, int32_t n_parts, int64_t n4,
                                                                  int32_t pieces) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * MERGE_THREADS;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * MERGE_THREADS + threadIdx.x; i < n4; i += stride) {
    const int64_t rh = i / pieces;
    float mx = -__builtin_inff();
    for (int p = 0; p < n_parts; ++p) mx = fmaxf(mx, parts.lse[p][rh]);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    if (mx != -__builtin_inff()) {
      // eight partials at a time: all their 16-byte loads are requested before the first one is used,
      // so a thread keeps eight loads in flight instead of one behind a dependent chain
      for (int p0 = 0; p0 < n_parts; p0 += 8) {
        f32x4 b[8];
        float w[8];
        // the lse values first (their second read hits the cache): vector memory loads complete in
        // order, so waiting for them afterwards would wait for the 16-byte loads issued before
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = parts.lse[p0 + k < n_parts ? p0 + k : n_parts - 1][rh];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int p = p0 + k < n_parts ? p0 + k : n_parts - 1;        // a repeat of the last one, weight 0
          b[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(parts.o[p]) + i);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = p0 + k < n_parts ? __expf(w[k] - mx) : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          den += w[k];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(w[k], b[k][e], acc[e]);
        }
      }
      const float rden = 1.f / den;
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] *= rden;
    }
    reinterpret_cast<f32x4*>(o_out)[i] = acc;
    // all pieces of a (row, head) sit in one wavefront (d/4 divides 64): every lane has read its lse
    // values before this store, so lse_out may alias a partial
    if (i - rh * pieces == 0) lse_out[rh] = mx != -__builtin_inff() ? mx + __logf(den) : mx;
  }
}

__global__ __launch_bounds__(MERGE_THREADS) void fill_empty_kernel(float* __restrict__ o, float* __restrict__ lse,
                                                                  int64_t n4, int32_t pieces, int64_t bstride_rh) {
  o += static_cast<int64_t>(blockIdx.y) * bstride_rh * pieces * 4;
  lse += static_cast<int64_t>(blockIdx.y) * bstride_rh;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * MERGE_THREADS;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * MERGE_THREADS + threadIdx.x; i < n4; i += stride) {
    reinterpret_cast<f32x4*>(o)[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i % pieces == 0) lse[i / pieces] = -__builtin_inff();
  }
}

__global__ __launch_bounds__(MERGE_THREADS) void cast_bf16_kernel(const float* __restrict__ src, __bf16* __restrict__ dst,
                                                                 int64_t n4) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * MERGE_THREADS;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * MERGE_THREADS + threadIdx.x; i < n4; i += stride) {
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src) + i);
    bf16x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = static_cast<__bf16>(a[e]);   // round to nearest even
    reinterpret_cast<bf16x4*>(dst)[i] = r;
  }
}

// Plain 16-byte copy, used to calibrate the HBM traffic counters against a transfer of known size.
__global__ __launch_bounds__(MERGE_THREADS) void copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                            int64_t n4) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * MERGE_THREADS;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * MERGE_THREADS + threadIdx.x; i < n4; i += stride)
    dst[i] = __builtin_nontemporal_load(src + i);
}

unsigned grid_for(int64_t n_items) {
  const int64_t want = (n_items + MERGE_THREADS - 1) / MERGE_THREADS;
  const int64_t cap = 256 * 32;                     // 32 resident workgroups' worth per CU is plenty
  return static_cast<unsigned>(want < 1 ? 1 : (want > cap ? cap : want));
}

}  // namespace merge_detail

hipError_t launch_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                        int64_t row0, int64_t rows, int32_t heads, int32_t d, int32_t batch, int64_t L,
                        hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (rows == L) { rows *= batch; batch = 1; }       // whole sequences: one contiguous range
  if (batch < 1 || batch > 65535) return hipErrorInvalidValue;
  const int64_t n4 = rows * heads * (d / 4), off = row0 * heads;
  // one launch for the whole batch: the second grid dimension walks the sequences
  return TASP_LAUNCH(merge_kernel, dim3(grid_for(n4), static_cast<unsigned>(batch)), dim3(MERGE_THREADS), stream,
                     o_acc + off * d, lse_acc + off, o_part + off * d, lse_part + off, n4, d / 4, L * heads);
}

hipError_t launch_fill_empty(float* o, float* lse, int64_t row0, int64_t rows, int32_t heads, int32_t d,
                             int32_t batch, int64_t L, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (rows == L) { rows *= batch; batch = 1; }
  if (batch < 1 || batch > 65535) return hipErrorInvalidValue;
  const int64_t n4 = rows * heads * (d / 4), off = row0 * heads;
  return TASP_LAUNCH(fill_empty_kernel, dim3(grid_for(n4), static_cast<unsigned>(batch)), dim3(MERGE_THREADS), stream,
                     o + off * d, lse + off, n4, d / 4, L * heads);
}

hipError_t launch_cast_bf16(const float* src, void* dst, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int64_t n4 = n / 4;
  return TASP_LAUNCH(cast_bf16_kernel, dim3(grid_for(n4)), dim3(MERGE_THREADS), stream, src,
                     static_cast<__bf16*>(dst), n4);
}

namespace {
constexpr int kI32PerLaunch = 896;
struct I32Chunk {
  int32_t n;
  int32_t v[kI32PerLaunch];
};
__global__ __launch_bounds__(256) void write_i32_kernel(int32_t* __restrict__ dst, const I32Chunk c) {
  for (int i = threadIdx.x; i < c.n; i += 256) dst[i] = c.v[i];
}
}  // namespace

hipError_t launch_write_i32(int32_t* dst, const int32_t* host_vals, int64_t n, hipStream_t stream) {
  for (int64_t i0 = 0; i0 < n; i0 += kI32PerLaunch) {
    I32Chunk c{};
    c.n = static_cast<int32_t>(n - i0 < kI32PerLaunch ? n - i0 : kI32PerLaunch);
    for (int i = 0; i < c.n; ++i) c.v[i] = host_vals[i0 + i];
    const hipError_t e = TASP_LAUNCH(write_i32_kernel, dim3(1), dim3(256), stream, dst + i0, c);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace tasp

extern "C" int tasp_calibration_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (bytes == 0) return TASP_OK;
  if (dst == nullptr || src == nullptr || bytes % 16 != 0) return TASP_EINVAL;
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15) return TASP_EALIGN;
  const int64_t n4 = static_cast<int64_t>(bytes / 16);
  const hipError_t e = TASP_LAUNCH(tasp::copy_kernel, dim3(tasp::grid_for(n4)), dim3(tasp::MERGE_THREADS),
                                   static_cast<hipStream_t>(hip_stream), static_cast<const tasp::f32x4*>(src),
                                   static_cast<tasp::f32x4*>(dst), n4);
  return e == hipSuccess ? TASP_OK : TASP_EHIP;
}

extern "C" int tasp_lse_merge_many(float* o_out, float* lse_out, const float* const* o_parts,
                                   const float* const* lse_parts, int32_t n_parts, int64_t rows, int32_t heads,
                                   int32_t d, void* hip_stream) {
  if (rows < 0 || heads <= 0 || d <= 0 || n_parts < 1 || n_parts > TASP_MAX_MERGE_PARTS) return TASP_EINVAL;
  if (d < 4 || d > 256 || (d & (d - 1)) != 0) return TASP_EUNSUPPORTED_SHAPE;
  if (rows == 0) return TASP_OK;
  if (o_out == nullptr || lse_out == nullptr || o_parts == nullptr || lse_parts == nullptr) return TASP_EINVAL;
  tasp::ManyParts parts{};
  uintptr_t bits16 = reinterpret_cast<uintptr_t>(o_out), bits4 = reinterpret_cast<uintptr_t>(lse_out);
  for (int p = 0; p < n_parts; ++p) {
    if (o_parts[p] == nullptr || lse_parts[p] == nullptr) return TASP_EINVAL;
    parts.o[p] = o_parts[p];
    parts.lse[p] = lse_parts[p];
    bits16 |= reinterpret_cast<uintptr_t>(o_parts[p]);
    bits4 |= reinterpret_cast<uintptr_t>(lse_parts[p]);
  }
  if ((bits16 & 15) || (bits4 & 3)) return TASP_EALIGN;
  const int64_t n4 = rows * heads * (d / 4);
  const hipError_t e = TASP_LAUNCH(tasp::merge_many_kernel, dim3(tasp::grid_for(n4)), dim3(tasp::MERGE_THREADS),
                                   static_cast<hipStream_t>(hip_stream), o_out, lse_out, parts, n_parts, n4, d / 4);
  return e == hipSuccess ? TASP_OK : TASP_EHIP;
}

extern "C" int tasp_lse_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                              int64_t rows, int32_t heads, int32_t d, void* hip_stream) {
  if (rows < 0 || heads <= 0 || d <= 0) return TASP_EINVAL;
  if (d < 4 || d > 256 || (d & (d - 1)) != 0) return TASP_EUNSUPPORTED_SHAPE;
  if (rows == 0) return TASP_OK;
  if (o_acc == nullptr || lse_acc == nullptr || o_part == nullptr || lse_part == nullptr) return TASP_EINVAL;
  if ((reinterpret_cast<uintptr_t>(o_acc) | reinterpret_cast<uintptr_t>(o_part)) & 15) return TASP_EALIGN;
  if ((reinterpret_cast<uintptr_t>(lse_acc) | reinterpret_cast<uintptr_t>(lse_part)) & 3) return TASP_EALIGN;
  const hipError_t e = tasp::launch_merge(o_acc, lse_acc, o_part, lse_part, 0, rows, heads, d, 1, rows,
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? TASP_OK : TASP_EHIP;
}
