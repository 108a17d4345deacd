// Blockwise attention of one step of Algorithm 3 for fp32 inputs (all arithmetic in fp32).
//
// This is the small-shape path (the fp32 workload is 256 local rows against 1024 keys): one
// wavefront owns one (query row, head).  Keys are taken 64 at a time, one key per lane; the scores
// of a chunk are reduced to the running max and sum with wavefront-level butterfly exchanges, and
// the output is accumulated with one lane per output column.
#include <hip/hip_runtime.h>

#include "internal.hpp"

namespace tasp {
namespace {

constexpr int WAVES = 4;

__device__ inline float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

template <int D>
__global__ __launch_bounds__(WAVES * 64) void attn_fp32_kernel(const AttnLaunch p) {
  constexpr int CPL = D / 64;                        // output columns per lane
  __shared__ float s_q[WAVES][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t item = static_cast<int64_t>(blockIdx.x) * WAVES + wave;   // (task row, head)
  int tsk = 0;
  const int64_t items0 = static_cast<int64_t>(p.task[0].n_q) * p.Hq;
  if (item >= items0) { item -= items0; tsk = 1; }
  if (tsk >= p.n_tasks) return;
  const AttnTask& T = p.task[tsk];
  if (item >= static_cast<int64_t>(T.n_q) * p.Hq) return;
  const int r = static_cast<int>(item / p.Hq), hq = static_cast<int>(item % p.Hq);
  const int g = hq / (p.Hq / p.Hkv);
  const int64_t row = T.q_row0 + r;
  const int q_pos = T.q_pos0 + r;
  const int64_t bi = blockIdx.y;                     // sequence of the batch
  const float* Qg = static_cast<const float*>(p.q) + bi * p.q_bstride + (row * p.Hq + hq) * D;
  const float* Kg = static_cast<const float*>(p.k) + bi * p.kv_bstride + static_cast<int64_t>(g) * D;
  const float* Vg = static_cast<const float*>(p.v) + bi * p.kv_bstride + static_cast<int64_t>(g) * D;
  const int64_t kv_stride = static_cast<int64_t>(p.Hkv) * D;
#pragma unroll
  for (int c = 0; c < CPL; ++c) s_q[wave][lane + 64 * c] = Qg[lane + 64 * c];
  __builtin_amdgcn_wave_barrier();

  float m = -__builtin_inff(), l = 0.f;
  float acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

  // with all steps in one launch the list comes from device memory; the running max / sum / output
  // simply carry on across the steps
  const int32_t* ext = p.seg_ext[tsk];
  for (int s = 0; s < T.n_seg; ++s) {
    const int a = ext != nullptr ? ext[2 * s] : T.seg_start[s];
    int b = ext != nullptr ? ext[2 * s + 1] : T.seg_end[s];
    if (p.causal) b = min(b, q_pos + 1);             // key t is visible iff t <= q_pos
    for (int t0 = a; t0 < b; t0 += 64) {
      const int t = t0 + lane;
      const bool valid = t < b;
      float sc = -__builtin_inff();
      if (valid) {
        const float4* kr = reinterpret_cast<const float4*>(Kg + t * kv_stride);
        float dot = 0.f;
#pragma unroll 4
        for (int c4 = 0; c4 < D / 4; ++c4) {
          const float4 kk = kr[c4];
          dot = fmaf(s_q[wave][4 * c4 + 0], kk.x, dot);
          dot = fmaf(s_q[wave][4 * c4 + 1], kk.y, dot);
          dot = fmaf(s_q[wave][4 * c4 + 2], kk.z, dot);
          dot = fmaf(s_q[wave][4 * c4 + 3], kk.w, dot);
        }
        sc = dot * p.scale;
      }
      const float m_new = fmaxf(m, wave_max(sc));    // finite: lane 0 of the chunk is always valid
      const float alpha = expf(m - m_new);           // exp(-inf) = 0 on the first chunk
      const float pr = valid ? expf(sc - m_new) : 0.f;
      l = l * alpha + wave_sum(pr);
#pragma unroll
      for (int c = 0; c < CPL; ++c) acc[c] *= alpha;
      const int n_here = min(64, b - t0);
      for (int j = 0; j < n_here; ++j) {
        const float pj = __shfl(pr, j);
        const float* vr = Vg + static_cast<int64_t>(t0 + j) * kv_stride;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] = fmaf(pj, vr[lane + 64 * c], acc[c]);
      }
      m = m_new;
    }
  }

  const bool seen = l > 0.f;
  const float inv = seen ? 1.f / l : 0.f;
  float lse_new = seen ? m + logf(l) : -__builtin_inff();
  float* od = p.o_dst + bi * p.o_bstride + (row * p.Hq + hq) * D;
  float* ld = p.lse_dst + bi * p.lse_bstride + row * p.Hq + hq;
  float wa = 0.f, wb = 1.f;
  if (p.merge) {                                     // update_out_lse of Algorithm 3
    const float lse_old = *ld;
    const float mx = fmaxf(lse_old, lse_new);
    if (mx == -__builtin_inff()) {
      wa = 0.f; wb = 0.f;
    } else {
      const float ea = expf(lse_old - mx), eb = expf(lse_new - mx);
      wa = ea / (ea + eb); wb = eb / (ea + eb);
      lse_new = mx + logf(ea + eb);
    }
  }
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    float val = acc[c] * inv * wb;
    if (p.merge) val += wa * od[lane + 64 * c];
    od[lane + 64 * c] = val;
  }
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) *ld = lse_new;
}

}  // namespace

hipError_t launch_attn_fp32(const AttnLaunch& p, int d, hipStream_t stream) {
  int64_t items = 0;
  for (int t = 0; t < p.n_tasks; ++t) items += static_cast<int64_t>(p.task[t].n_q) * p.Hq;
  if (items == 0) return hipSuccess;
  const int64_t blocks = (items + WAVES - 1) / WAVES;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  if (p.batch < 1 || p.batch > 65535) return hipErrorInvalidValue;
  dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(p.batch)), block(WAVES * 64);
  if (d == 64) return TASP_LAUNCH(attn_fp32_kernel<64>, grid, block, stream, p);
  if (d == 128) return TASP_LAUNCH(attn_fp32_kernel<128>, grid, block, stream, p);
  return hipErrorInvalidValue;
}

}  // namespace tasp
