// Backward pass of one step of the chunked attention for fp32 inputs (all arithmetic in fp32).
//
// Small-shape path like the fp32 forward kernel, not tuned: one wavefront owns one query row and
// head (dq) or one key and KV head (dk, dv), holds its own row with one lane per column, and walks
// the other side one row at a time; the two dot products of a pair (scores, dout.v) are wavefront
// sums.  The formulas are those of the bf16 kernels:
//   p = exp(scale q.k - lse),  ds = p (dout.v - delta),  dq += scale ds k,  dk += scale ds q,  dv += p dout.
#include <hip/hip_runtime.h>

#include <climits>

#include "internal.hpp"

namespace tasp {
namespace {

constexpr int WAVES = 4;

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

template <int D>
__global__ __launch_bounds__(WAVES * 64) void bwd_dq_fp32_kernel(const BwdLaunch p) {
  constexpr int CPL = D / 64;                        // columns per lane
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
  const int64_t bi = blockIdx.y;
  const int64_t qoff = bi * p.q_bstride + (row * p.Hq + hq) * D;
  const float* Kg = static_cast<const float*>(p.k) + bi * p.kv_bstride + static_cast<int64_t>(g) * D;
  const float* Vg = static_cast<const float*>(p.v) + bi * p.kv_bstride + static_cast<int64_t>(g) * D;
  const int64_t kv_stride = static_cast<int64_t>(p.Hkv) * D;
  const float lse = p.lse[bi * p.lse_bstride + row * p.Hq + hq];
  const float dl = p.delta[bi * p.lse_bstride + row * p.Hq + hq];
  if (!(lse > -__builtin_inff())) return;            // the row saw no key: nothing to add
  float q[CPL], go[CPL], acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    q[c] = static_cast<const float*>(p.q)[qoff + lane + 64 * c];
    go[c] = static_cast<const float*>(p.dout)[qoff + lane + 64 * c];
    acc[c] = 0.f;
  }
  for (int s = 0; s < T.n_seg; ++s) {
    const int a = T.seg_start[s];
    int b = T.seg_end[s];
    if (p.causal) b = min(b, q_pos + 1);             // key t is visible iff t <= q_pos
    for (int t = a; t < b; ++t) {
      float kx[CPL], sk = 0.f, sv = 0.f;
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        kx[c] = Kg[t * kv_stride + lane + 64 * c];
        sk = __builtin_fmaf(q[c], kx[c], sk);
        sv = __builtin_fmaf(go[c], Vg[t * kv_stride + lane + 64 * c], sv);
      }
      const float pr = __expf(wave_sum(sk) * p.scale - lse);
      const float ds = pr * (wave_sum(sv) - dl);
#pragma unroll
      for (int c = 0; c < CPL; ++c) acc[c] = __builtin_fmaf(ds, kx[c], acc[c]);
    }
  }
  float* dq = p.dq_acc + qoff;
#pragma unroll
  for (int c = 0; c < CPL; ++c) dq[lane + 64 * c] += acc[c] * p.scale;
}

template <int D>
__global__ __launch_bounds__(WAVES * 64) void bwd_dkv_fp32_kernel(const BwdLaunch p) {
  constexpr int CPL = D / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t item = static_cast<int64_t>(blockIdx.x) * WAVES + wave;   // (key of the step, KV head)
  const int total_keys = p.rng_vbeg[p.n_rng];
  if (item >= static_cast<int64_t>(total_keys) * p.Hkv) return;
  const int vi = static_cast<int>(item / p.Hkv), g = static_cast<int>(item % p.Hkv);
  int tok = 0;
  for (int j = 0; j < p.n_rng; ++j)
    if (vi >= p.rng_vbeg[j] && vi < p.rng_vbeg[j + 1]) tok = p.rng_start[j] + (vi - p.rng_vbeg[j]);
  const int G = p.Hq / p.Hkv;
  const int64_t bi = blockIdx.y;
  const int64_t koff = bi * p.kv_bstride + (static_cast<int64_t>(tok) * p.Hkv + g) * D;
  float kx[CPL], vx[CPL], dk[CPL], dv[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    kx[c] = static_cast<const float*>(p.k)[koff + lane + 64 * c];
    vx[c] = static_cast<const float*>(p.v)[koff + lane + 64 * c];
    dk[c] = dv[c] = 0.f;
  }
  const float* Qg = static_cast<const float*>(p.q) + bi * p.q_bstride;
  const float* Og = static_cast<const float*>(p.dout) + bi * p.q_bstride;
  for (int hh = 0; hh < G; ++hh) {
    const int hq = g * G + hh;
    for (int blk = 0; blk < p.n_blk; ++blk) {
      const BwdBlock& B = p.blk[blk];
      const int r0 = p.causal ? max(0, tok - B.pos0) : 0;        // the first row at or after the key
      for (int r = r0; r < B.n; ++r) {
        const int64_t row = B.row0 + r;
        const float lse = p.lse[bi * p.lse_bstride + row * p.Hq + hq];
        if (!(lse > -__builtin_inff())) continue;
        const float dl = p.delta[bi * p.lse_bstride + row * p.Hq + hq];
        float qx[CPL], gx[CPL], sk = 0.f, sv = 0.f;
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
          qx[c] = Qg[(row * p.Hq + hq) * D + lane + 64 * c];
          gx[c] = Og[(row * p.Hq + hq) * D + lane + 64 * c];
          sk = __builtin_fmaf(qx[c], kx[c], sk);
          sv = __builtin_fmaf(gx[c], vx[c], sv);
        }
        const float pr = __expf(wave_sum(sk) * p.scale - lse);
        const float ds = pr * (wave_sum(sv) - dl);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
          dv[c] = __builtin_fmaf(pr, gx[c], dv[c]);
          dk[c] = __builtin_fmaf(ds, qx[c], dk[c]);
        }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    static_cast<float*>(p.dk)[koff + lane + 64 * c] = dk[c] * p.scale;
    static_cast<float*>(p.dv)[koff + lane + 64 * c] = dv[c];
  }
}

template <int D>
__global__ __launch_bounds__(256) void bwd_delta_fp32_kernel(const float* __restrict__ out, const float* __restrict__ dout,
                                                             float* __restrict__ delta, int64_t n_rows) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < D / 64; ++c) s = __builtin_fmaf(out[row * D + lane + 64 * c], dout[row * D + lane + 64 * c], s);
  s = wave_sum(s);
  if (lane == 0) delta[row] = s;
}

}  // namespace

hipError_t launch_bwd_dq_fp32(const BwdLaunch& p, int d, hipStream_t stream) {
  int64_t items = 0;
  for (int t = 0; t < p.n_tasks; ++t) items += static_cast<int64_t>(p.task[t].n_q) * p.Hq;
  const int64_t blocks = (items + WAVES - 1) / WAVES;
  if (blocks == 0) return hipSuccess;
  if (blocks > INT_MAX || p.batch > 65535) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(p.batch));
  if (d == 128) return TASP_LAUNCH((bwd_dq_fp32_kernel<128>), grid, dim3(WAVES * 64), stream, p);
  if (d == 64) return TASP_LAUNCH((bwd_dq_fp32_kernel<64>), grid, dim3(WAVES * 64), stream, p);
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_dkv_fp32(const BwdLaunch& p, int d, hipStream_t stream) {
  const int64_t items = static_cast<int64_t>(p.rng_vbeg[p.n_rng]) * p.Hkv;
  const int64_t blocks = (items + WAVES - 1) / WAVES;
  if (blocks == 0) return hipSuccess;
  if (blocks > INT_MAX || p.batch > 65535) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(p.batch));
  if (d == 128) return TASP_LAUNCH((bwd_dkv_fp32_kernel<128>), grid, dim3(WAVES * 64), stream, p);
  if (d == 64) return TASP_LAUNCH((bwd_dkv_fp32_kernel<64>), grid, dim3(WAVES * 64), stream, p);
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_delta_fp32(const void* out, const void* dout, float* delta, int64_t n_rows, int d,
                                 hipStream_t stream) {
  if (n_rows == 0) return hipSuccess;
  const int64_t blocks = (n_rows + 3) / 4;
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  const float* o = static_cast<const float*>(out);
  const float* g = static_cast<const float*>(dout);
  if (d == 128) return TASP_LAUNCH((bwd_delta_fp32_kernel<128>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, o, g, delta, n_rows);
  if (d == 64) return TASP_LAUNCH((bwd_delta_fp32_kernel<64>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, o, g, delta, n_rows);
  return hipErrorInvalidValue;
}

}  // namespace tasp
