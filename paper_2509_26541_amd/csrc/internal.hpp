// Launch descriptors shared by the host orchestration and the kernels of this library.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace tasp {

constexpr int kMaxSeg = 64;      // KV segments one query block can see in one step (2(N-1) for zig-zag)
constexpr int kMaxTasks = 2;     // query blocks per step (the two half-chunks of the zig-zag layout)
constexpr int kMaxSegAll = 1024; // segments of one query block over ALL steps (single-launch mode)

// One query block of one step: rows [q_row0, q_row0 + n_q) of the local Q, contiguous in the
// sequence from q_pos0, attending to the concatenation of seg[0..n_seg).
struct AttnTask {
  int32_t q_row0;
  int32_t n_q;
  int32_t q_pos0;
  int32_t n_seg;
  int32_t seg_start[kMaxSeg];
  int32_t seg_end[kMaxSeg];
};

struct AttnLaunch {
  const void* q;      // [L, Hq, d]
  const void* k;      // [S, Hkv, d]
  const void* v;      // [S, Hkv, d]
  float* o_dst;       // [L, Hq, d] fp32
  float* lse_dst;     // [L, Hq]    fp32
  int32_t Hq, Hkv;
  int32_t causal;     // key t visible to query p iff t <= p
  int32_t merge;      // 0: dst = partial of this step; 1: dst = update_out_lse(dst, partial)
  float scale;        // softmax scale (natural units)
  int32_t batch;      // independent sequences; element strides between them:
  int64_t q_bstride, kv_bstride, o_bstride, lse_bstride;
  int32_t n_tasks;
  AttnTask task[kMaxTasks];
  // Single-launch mode: the segment list of task t does not fit the descriptor and lives in device
  // memory as task[t].n_seg (start, end) pairs; task[t].seg_start / seg_end are then unused.
  const int32_t* seg_ext[kMaxTasks];
  int32_t n_items;    // work items of the launch, for persistent workgroups; filled in by the launcher
};

// One contiguous run of local query rows (a half-chunk of the zig-zag layout, or all rows).
struct BwdBlock {
  int32_t row0, n, pos0;   // first local row, rows, global position of the first row
};

// One step of the backward pass.  The dq kernel uses the forward's tasks (query block + the key
// segments it can see); the dk/dv kernel uses every key range that arrives at the step, laid end to
// end (rng_vbeg = start of each range in that concatenation), and the query blocks.
struct BwdLaunch {
  const void* q;        // [B, L, Hq, d] bf16 (fp32 for the fp32 kernels, as k, v, dout, dk, dv)
  const void* k;        // [B, S, Hkv, d]
  const void* v;
  const void* dout;     // [B, L, Hq, d]
  const float* lse;     // [B, L, Hq] final lse of the forward pass
  const float* delta;   // [B, L, Hq] sum_d dout * out (fp32 kernels)
  const float* ndelta;  // [B, L, Hq] -delta, then one 0 (bf16 kernels)
  const float* nlse;    // [B, L, Hq] -lse / scale, -inf where lse is -inf (the row saw no key), then one -inf (bf16 kernels)
  float* dq_acc;        // [B, L, Hq, d] fp32, accumulated into
  void* dk;             // [B, S, Hkv, d] bf16; the rows of this step's keys are written
  void* dv;
  int32_t Hq, Hkv;
  int32_t causal;
  float scale;
  int32_t batch;
  int64_t q_bstride, kv_bstride, lse_bstride;   // elements between sequences
  int32_t n_tasks;
  AttnTask task[kMaxTasks];
  const int32_t* seg_ext[kMaxTasks];   // as in AttnLaunch (all steps in one launch)
  int32_t n_blk;
  BwdBlock blk[kMaxTasks];
  int32_t n_rng;
  int32_t rng_start[kMaxSeg];
  int32_t rng_vbeg[kMaxSeg + 1];
  // dk/dv launch split by query head (a workgroup per key tile AND query head of the group, for
  // launches whose key tiles alone are too few and too unequal to fill the chip): the workgroups
  // write fp32 partial sums [B, Hq / Hkv, keys of the launch, Hkv, d] (unscaled, keys in the order of
  // the concatenated ranges) and launch_bwd_dkv_reduce adds them up in a fixed order.
  int32_t split_heads;
  float* part_dk;
  float* part_dv;
};

// Last HIP error this thread saw inside the library (hipSuccess if none); see tasp_last_hip_error().
extern thread_local hipError_t g_last_hip_error;
inline hipError_t note_hip(hipError_t e) {
  if (e != hipSuccess) g_last_hip_error = e;
  return e;
}

// Launch with a clean error slot: an error left behind by an earlier, unrelated HIP call in this
// thread must not be mistaken for a failure of this launch.
#define TASP_LAUNCH(kernel, grid, block, stream, ...)                         \
  ({                                                                          \
    (void)hipGetLastError();                                                  \
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);          \
    ::tasp::note_hip(hipGetLastError());                                      \
  })

// Implemented in attn_bf16.hip / attn_fp32.hip / merge.hip.  Each returns a hipError_t from the launch.
hipError_t launch_attn_bf16(const AttnLaunch& p, int d, hipStream_t stream);
hipError_t launch_attn_fp32(const AttnLaunch& p, int d, hipStream_t stream);
// rows [row0, row0 + rows) of every one of `batch` sequences of L rows each
hipError_t launch_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                        int64_t row0, int64_t rows, int32_t heads, int32_t d, int32_t batch, int64_t L,
                        hipStream_t stream);
hipError_t launch_fill_empty(float* o, float* lse, int64_t row0, int64_t rows, int32_t heads, int32_t d,
                             int32_t batch, int64_t L, hipStream_t stream);
hipError_t launch_cast_bf16(const float* src, void* dst, int64_t n, hipStream_t stream);
// Writes n host integers to device memory with small kernels that carry them as arguments (no copy
// from host memory is enqueued, so the call can be recorded into a graph).
hipError_t launch_write_i32(int32_t* dst, const int32_t* host_vals, int64_t n, hipStream_t stream);
// Implemented in attn_bwd_bf16.hip.
hipError_t launch_bwd_dq_bf16(const BwdLaunch& p, int d, hipStream_t stream);
hipError_t launch_bwd_dkv_bf16(const BwdLaunch& p, int d, hipStream_t stream);
// after a launch with split_heads: dk, dv = sum over the query heads of the partial sums, as bf16
hipError_t launch_bwd_dkv_reduce(const BwdLaunch& p, int d, hipStream_t stream);
// workgroups of the dk/dv launch without the split, and how many of them the chip holds at once
int64_t bwd_dkv_workgroups(const BwdLaunch& p, int d);
int bwd_dkv_resident_workgroups(int d);
// ndelta[r] = -sum_d dout out and nlse[r] = -lse[r] / scale (-inf for -inf) for the n_rows (row, head)
// pairs; both arrays hold n_rows + 1 floats, the last one being 0 and -inf.
hipError_t launch_bwd_delta_bf16(const void* out, const void* dout, const float* lse, float* ndelta, float* nlse,
                                 float scale, int64_t n_rows, int d, hipStream_t stream);
hipError_t launch_zero_f32(float* dst, int64_t n, hipStream_t stream);   // n a multiple of 4, dst 16-byte aligned
// Implemented in attn_bwd_fp32.hip (all tensors fp32; dq_acc is dq itself).
hipError_t launch_bwd_dq_fp32(const BwdLaunch& p, int d, hipStream_t stream);
hipError_t launch_bwd_dkv_fp32(const BwdLaunch& p, int d, hipStream_t stream);
hipError_t launch_bwd_delta_fp32(const void* out, const void* dout, float* delta, int64_t n_rows, int d,
                                 hipStream_t stream);

}  // namespace tasp
