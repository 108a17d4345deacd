// Host orchestration of one rank's forward pass (Algorithm 3): N steps, each one attention launch
// over the sub-chunks the schedule delivers at that step, followed by update_out_lse; and of the
// backward pass, which walks the same steps in the same order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <functional>
#include <mutex>
#include <vector>

#include "internal.hpp"
#include "schedule.hpp"
#include "tasp.h"

// Scratch of tasp_chunk_attn_static: the workspace of a forward call, held in the code object instead
// of being brought in by the caller.  In host code this name is only a handle for the HIP symbol
// query below; the address the kernels get is the one that query returns, per device.
static __device__ __align__(256) unsigned char scratch[TASP_STATIC_SCRATCH_BYTES];

namespace {

using tasp::AttnLaunch;
using tasp::AttnTask;

constexpr size_t kAlign = 256;
constexpr size_t kFusedTableBytes = static_cast<size_t>(tasp::kMaxTasks) * 2 * tasp::kMaxSegAll * sizeof(int32_t);
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Shape {
  int64_t L;            // local rows of one sequence
  int32_t B;            // sequences in the batch
  size_t o_bytes;       // fp32 [B, L, Hq, d]
  size_t lse_bytes;     // fp32 [B, L, Hq]
};

int32_t batch_of(const tasp_attn_args* a) { return a->batch == 0 ? 1 : a->batch; }

int validate(const tasp_schedule_t* s, const tasp_attn_args* a, Shape* sh) {
  if (s == nullptr || a == nullptr) return TASP_EINVAL;
  if (a->q == nullptr || a->k == nullptr || a->v == nullptr) return TASP_EINVAL;
  int st = tasp::check_sequence(*s, a->S, a->mask_mode);
  if (st != TASP_OK) return st;
  if (a->Hq <= 0 || a->Hkv <= 0 || a->Hq % a->Hkv != 0) return TASP_EINVAL;
  if (a->order != TASP_ORDER_TASP && a->order != TASP_ORDER_RING) return TASP_EINVAL;
  if (!(a->softmax_scale >= 0.f) || !std::isfinite(a->softmax_scale)) return TASP_EINVAL;
  if (a->dtype != TASP_DTYPE_FP32 && a->dtype != TASP_DTYPE_BF16) return TASP_EUNSUPPORTED_SHAPE;
  if (a->d != 64 && a->d != 128) return TASP_EUNSUPPORTED_SHAPE;
  if (a->S >= (int64_t{1} << 31) - 4096) return TASP_EUNSUPPORTED_SHAPE;
  if (a->dtype == TASP_DTYPE_BF16) {
    // the bf16 kernel addresses K and V with 32-bit byte offsets formed by a 24-bit multiply
    const int64_t row_bytes = static_cast<int64_t>(a->Hkv) * a->d * 2;
    if (a->S >= (1 << 24) || row_bytes >= (1 << 24) || a->S * row_bytes > (int64_t{1} << 32))
      return TASP_EUNSUPPORTED_SHAPE;
    // the forward kernel reads them through buffer descriptors of 2^32 - 1 bytes that start at the
    // KV head's first row: only with a single KV head can the last row end at 2^32 exactly
    if (a->Hkv == 1 && a->S * row_bytes == (int64_t{1} << 32)) return TASP_EUNSUPPORTED_SHAPE;
  }
  if (2 * s->n_rings > tasp::kMaxSeg) return TASP_EUNSUPPORTED_SHAPE;
  if (a->batch < 0 || a->batch > 65535) return TASP_EINVAL;
  if (a->fuse_steps != 0 && a->fuse_steps != 1) return TASP_EINVAL;
  if ((reinterpret_cast<uintptr_t>(a->q) | reinterpret_cast<uintptr_t>(a->k) | reinterpret_cast<uintptr_t>(a->v)) & 15)
    return TASP_EALIGN;
  sh->L = a->S / s->n;
  sh->B = batch_of(a);
  sh->o_bytes = static_cast<size_t>(sh->B) * sh->L * a->Hq * a->d * sizeof(float);
  sh->lse_bytes = static_cast<size_t>(sh->B) * sh->L * a->Hq * sizeof(float);
  return TASP_OK;
}

// Builds the launch descriptor of one step; `empty` receives the query blocks that see no key.
int build_step(const tasp_schedule_t* s, const tasp_attn_args* a, int step, AttnLaunch* lp,
               std::vector<tasp::QueryBlock>* empty) {
  lp->q = a->q; lp->k = a->k; lp->v = a->v;
  lp->Hq = a->Hq; lp->Hkv = a->Hkv;
  lp->causal = a->mask_mode == TASP_MASK_ZIGZAG_CAUSAL ? 1 : 0;
  lp->scale = a->softmax_scale > 0.f ? a->softmax_scale : 1.0f / std::sqrt(static_cast<float>(a->d));
  const int64_t L = a->S / s->n;
  lp->batch = batch_of(a);
  lp->q_bstride = L * a->Hq * a->d;
  lp->kv_bstride = a->S * a->Hkv * a->d;
  lp->o_bstride = L * a->Hq * a->d;
  lp->lse_bstride = L * a->Hq;
  lp->n_tasks = 0;
  int64_t keys[tasp::kMaxTasks] = {0, 0};
  std::vector<tasp::Segment> segs;
  for (int qb = 0; qb < tasp::n_query_blocks(a->mask_mode); ++qb) {
    tasp::QueryBlock blk;
    int st = tasp::query_block(*s, a->S, a->mask_mode, qb, &blk);
    if (st != TASP_OK) return st;
    st = tasp::step_segments(*s, a->S, a->mask_mode, a->order, step, qb, &segs);
    if (st != TASP_OK) return st;
    if (segs.empty()) { empty->push_back(blk); continue; }
    if (segs.size() > static_cast<size_t>(tasp::kMaxSeg)) return TASP_EUNSUPPORTED_SHAPE;
    AttnTask& t = lp->task[lp->n_tasks];
    t.q_row0 = static_cast<int32_t>(blk.local_row0);
    t.n_q = static_cast<int32_t>(blk.rows);
    t.q_pos0 = static_cast<int32_t>(blk.pos0);
    t.n_seg = static_cast<int32_t>(segs.size());
    int64_t total = 0;
    for (size_t i = 0; i < segs.size(); ++i) {
      t.seg_start[i] = static_cast<int32_t>(segs[i].start);
      t.seg_end[i] = static_cast<int32_t>(segs[i].end);
      total += segs[i].end - segs[i].start;
    }
    keys[lp->n_tasks++] = total;
  }
  // the block with more keys goes first so that its workgroups are not the tail of the launch
  if (lp->n_tasks == 2 && keys[1] > keys[0]) std::swap(lp->task[0], lp->task[1]);
  return TASP_OK;
}

// Single-launch mode: the tasks of all steps joined per query block, in arrival order.  The segment
// lists go to `dev_table` (kMaxTasks x 2 kMaxSegAll integers of device memory, written by small
// kernels on `stream`); the descriptor points at them.
int build_all_steps(const tasp_schedule_t* s, const tasp_attn_args* a, int32_t* dev_table, hipStream_t stream,
                    AttnLaunch* all) {
  std::vector<int32_t> table[tasp::kMaxTasks];
  std::vector<tasp::QueryBlock> empty;
  int64_t keys[tasp::kMaxTasks] = {0, 0};
  for (int step = 0; step < s->n; ++step) {
    AttnLaunch lp{};
    empty.clear();
    const int st = build_step(s, a, step, &lp, &empty);
    if (st != TASP_OK) return st;
    if (step == 0) {
      // every query block sees its own diagonal at step 0, so step 0 defines the blocks
      if (!empty.empty()) return TASP_EUNSUPPORTED_SHAPE;
      *all = lp;
      for (int t = 0; t < all->n_tasks; ++t) all->task[t].n_seg = 0;
    }
    for (int t = 0; t < lp.n_tasks; ++t) {
      int dst = -1;
      for (int u = 0; u < all->n_tasks; ++u)
        if (all->task[u].q_row0 == lp.task[t].q_row0) dst = u;
      if (dst < 0) return TASP_EUNSUPPORTED_SHAPE;
      for (int i = 0; i < lp.task[t].n_seg; ++i) {
        table[dst].push_back(lp.task[t].seg_start[i]);
        table[dst].push_back(lp.task[t].seg_end[i]);
        keys[dst] += lp.task[t].seg_end[i] - lp.task[t].seg_start[i];
      }
    }
  }
  for (int t = 0; t < all->n_tasks; ++t) {
    const size_t n_seg = table[t].size() / 2;
    if (n_seg > static_cast<size_t>(tasp::kMaxSegAll)) return TASP_EUNSUPPORTED_SHAPE;
    all->task[t].n_seg = static_cast<int32_t>(n_seg);
    all->seg_ext[t] = dev_table + static_cast<size_t>(t) * 2 * tasp::kMaxSegAll;
    if (tasp::launch_write_i32(dev_table + static_cast<size_t>(t) * 2 * tasp::kMaxSegAll, table[t].data(),
                               static_cast<int64_t>(table[t].size()), stream) != hipSuccess)
      return TASP_EHIP;
  }
  // the block with more keys goes first so that its workgroups are not the tail of the launch
  if (all->n_tasks == 2 && keys[1] > keys[0]) {
    std::swap(all->task[0], all->task[1]);
    std::swap(all->seg_ext[0], all->seg_ext[1]);
  }
  return TASP_OK;
}

// Optional per-launch timing with HIP events on the caller's stream (tasp_chunk_attn_profile).
struct Profiler {
  enum Kind { kAttn = 0, kMerge = 1, kOther = 2 };
  struct Span { int kind; hipEvent_t beg, end; };
  std::vector<Span> spans;
  hipStream_t stream = nullptr;
  bool failed = false;
  void begin(int kind) {
    if (failed) return;
    spans.push_back(Span{kind, nullptr, nullptr});       // pushed first: the destructor owns whatever gets created
    Span& sp = spans.back();
    if (hipEventCreate(&sp.beg) != hipSuccess || hipEventCreate(&sp.end) != hipSuccess ||
        hipEventRecord(sp.beg, stream) != hipSuccess)
      failed = true;
  }
  void end() {
    if (spans.empty() || failed) return;
    if (hipEventRecord(spans.back().end, stream) != hipSuccess) failed = true;
  }
  ~Profiler() {
    for (auto& sp : spans) {
      if (sp.beg) (void)hipEventDestroy(sp.beg);
      if (sp.end) (void)hipEventDestroy(sp.end);
    }
  }
};
struct Scope {
  Profiler* p;
  Scope(Profiler* prof, int kind) : p(prof) { if (p) p->begin(kind); }
  ~Scope() { if (p) p->end(); }
};

hipError_t launch_attn(const AttnLaunch& lp, const tasp_attn_args* a, hipStream_t stream) {
  if (lp.n_tasks == 0) return hipSuccess;
  return a->dtype == TASP_DTYPE_BF16 ? tasp::launch_attn_bf16(lp, a->d, stream)
                                     : tasp::launch_attn_fp32(lp, a->d, stream);
}

// ---- backward pass
// The forward's argument block with the fields both passes share, so that one validation serves both.
tasp_attn_args as_forward(const tasp_attn_bwd_args* b) {
  tasp_attn_args a{};
  a.q = b->q; a.k = b->k; a.v = b->v;
  a.S = b->S; a.Hq = b->Hq; a.Hkv = b->Hkv; a.d = b->d;
  a.dtype = b->dtype; a.mask_mode = b->mask_mode; a.order = b->order;
  a.fuse_merge = 1; a.softmax_scale = b->softmax_scale; a.batch = b->batch;
  a.fuse_steps = b->fuse_steps;
  return a;
}

int validate_bwd(const tasp_schedule_t* s, const tasp_attn_bwd_args* b, tasp_attn_args* a, Shape* sh) {
  if (s == nullptr || b == nullptr) return TASP_EINVAL;
  *a = as_forward(b);
  int st = validate(s, a, sh);
  if (st != TASP_OK) return st;
  if (b->fuse_steps && b->dtype != TASP_DTYPE_BF16) return TASP_EUNSUPPORTED_SHAPE;   // the plain fp32 backward path walks step by step
  if (b->out == nullptr || b->lse == nullptr || b->dout == nullptr || b->dq == nullptr || b->dk == nullptr ||
      b->dv == nullptr)
    return TASP_EINVAL;
  // the bf16 kernels address Q and dout with 32-bit byte offsets
  if (b->dtype == TASP_DTYPE_BF16 && static_cast<int64_t>(sh->L) * b->Hq * b->d * 2 > (int64_t{1} << 32))
    return TASP_EUNSUPPORTED_SHAPE;
  const uintptr_t all = reinterpret_cast<uintptr_t>(b->out) | reinterpret_cast<uintptr_t>(b->dout) |
                        reinterpret_cast<uintptr_t>(b->dq) | reinterpret_cast<uintptr_t>(b->dk) |
                        reinterpret_cast<uintptr_t>(b->dv);
  if (all & 15) return TASP_EALIGN;
  return TASP_OK;
}

struct BwdSpans { enum Kind { kDq = 0, kDkv = 1, kOther = 2 }; };

// Estimated duration of a dk/dv launch, in 64-row query tiles of one head, with one workgroup per
// key tile (`per_tile` = 1, each serving all G query heads of its group) or per key tile and query
// head (`per_tile` = G).  Mirrors what the kernel and the hardware do: the work list is (sequence,
// KV head, head, key tile) in that order, every XCD gets one contiguous eighth of it (exactly so when
// the KV heads of the call are a multiple of 8; otherwise XCDs share heads, which this estimate
// ignores), and each of its slots/8 workgroup slots takes the next workgroup when it is free.  A workgroup walks, for
// each query block, the tiles from the first one that holds a row at or after its first key.
int64_t dkv_makespan(const tasp::BwdLaunch& bp, int d, int per_tile, int slots) {
  const int bs = d == 128 ? 256 : 128, bt = 64;
  const int64_t total = bp.rng_vbeg[bp.n_rng];
  const int64_t ktiles = (total + bs - 1) / bs;
  const int G = bp.Hq / bp.Hkv;
  std::vector<int32_t> work(static_cast<size_t>(ktiles));
  int j = 0;
  for (int64_t t = 0; t < ktiles; ++t) {
    while (j + 1 < bp.n_rng && bp.rng_vbeg[j + 1] <= t * bs) ++j;     // the range that holds the tile's first key
    // ranges are sorted by position, so the tile's first key is its earliest
    const int64_t tmin = bp.rng_start[j] + (t * bs - bp.rng_vbeg[j]);
    int64_t w = 0;
    for (int qb = 0; qb < bp.n_blk; ++qb) {
      const int64_t tiles = (bp.blk[qb].n + bt - 1) / bt;
      const int64_t first = bp.causal ? std::max<int64_t>(0, (tmin - bp.blk[qb].pos0) / bt) : 0;
      w += std::max<int64_t>(0, tiles - first);
    }
    work[static_cast<size_t>(t)] = static_cast<int32_t>(w);
  }
  const int64_t n = ktiles * bp.Hkv * bp.batch * per_tile;
  const int xcd_slots = std::max(1, slots / 8);
  constexpr int64_t kFixed = 4;      // set-up and epilogue of a workgroup, in the same unit
  int64_t makespan = 0;
  std::vector<int64_t> heap;
  for (int x = 0; x < 8; ++x) {
    const int64_t q8 = n / 8, r8 = n % 8;
    const int64_t start = x * q8 + std::min<int64_t>(x, r8), cnt = q8 + (x < r8 ? 1 : 0);
    heap.assign(static_cast<size_t>(xcd_slots), 0);
    for (int64_t i = start; i < start + cnt; ++i) {
      const int64_t tile = i % ktiles;
      const int64_t w = kFixed + static_cast<int64_t>(work[static_cast<size_t>(tile)]) * (per_tile == 1 ? G : 1);
      std::pop_heap(heap.begin(), heap.end(), std::greater<int64_t>());
      heap.back() += w;
      std::push_heap(heap.begin(), heap.end(), std::greater<int64_t>());
    }
    makespan = std::max(makespan, *std::max_element(heap.begin(), heap.end()));
  }
  return makespan;
}

}  // namespace

namespace tasp {
thread_local hipError_t g_last_hip_error = hipSuccess;
}

extern "C" {

const char* tasp_last_hip_error(void) { return hipGetErrorString(tasp::g_last_hip_error); }

size_t tasp_chunk_attn_workspace_bytes(const tasp_schedule_t* s, const tasp_attn_args* a) {
  if (s == nullptr || a == nullptr || a->S <= 0 || a->Hq <= 0 || a->d <= 0 || s->n <= 0 || a->batch < 0) return 0;
  const int64_t L = a->S / s->n;
  const size_t B = static_cast<size_t>(batch_of(a));
  const size_t o_bytes = align_up(B * L * a->Hq * a->d * sizeof(float));
  const size_t lse_bytes = align_up(B * L * a->Hq * sizeof(float));
  size_t total = 0;
  if (a->dtype == TASP_DTYPE_BF16) total += o_bytes;              // running fp32 output
  if (a->fuse_steps) return total + align_up(kFusedTableBytes);   // the segment lists of the single launch
  if (!a->fuse_merge) total += o_bytes + lse_bytes;               // partial (out_s, lse_s) of a step
  return total;
}

double tasp_chunk_attn_flops(const tasp_schedule_t* s, const tasp_attn_args* a) {
  if (s == nullptr || a == nullptr) return 0.0;
  if (tasp::check_sequence(*s, a->S, a->mask_mode) != TASP_OK) return 0.0;
  double pairs = 0.0;
  for (int qb = 0; qb < tasp::n_query_blocks(a->mask_mode); ++qb) {
    tasp::QueryBlock blk;
    if (tasp::query_block(*s, a->S, a->mask_mode, qb, &blk) != TASP_OK) return 0.0;
    const double rows = static_cast<double>(blk.rows);
    if (a->mask_mode == TASP_MASK_FULL) pairs += rows * static_cast<double>(a->S);
    else pairs += rows * static_cast<double>(blk.pos0) + rows * (rows + 1.0) / 2.0;   // sum of (p + 1)
  }
  return 4.0 * a->d * a->Hq * pairs * (a->batch > 0 ? a->batch : 1);
}

int tasp_step_attn(const tasp_schedule_t* s, const tasp_attn_args* a, int32_t step, float* o_part,
                   float* lse_part, void* hip_stream) {
  Shape sh;
  int st = validate(s, a, &sh);
  if (st != TASP_OK) return st;
  if (o_part == nullptr || lse_part == nullptr || step < 0 || step >= s->n) return TASP_EINVAL;
  if (reinterpret_cast<uintptr_t>(o_part) & 15) return TASP_EALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  try {
    AttnLaunch lp{};
    std::vector<tasp::QueryBlock> empty;
    st = build_step(s, a, step, &lp, &empty);
    if (st != TASP_OK) return st;
    lp.o_dst = o_part; lp.lse_dst = lse_part; lp.merge = 0;
    if (launch_attn(lp, a, stream) != hipSuccess) return TASP_EHIP;
    for (const auto& blk : empty)
      if (tasp::launch_fill_empty(o_part, lse_part, blk.local_row0, blk.rows, a->Hq, a->d, sh.B, sh.L, stream) !=
          hipSuccess)
        return TASP_EHIP;
  } catch (...) {
    return TASP_ENOMEM;
  }
  return TASP_OK;
}

static int run_chunk_attn(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream, Profiler* prof) {
  Shape sh;
  int st = validate(s, a, &sh);
  if (st != TASP_OK) return st;
  if (a->out == nullptr || a->lse == nullptr) return TASP_EINVAL;
  if (reinterpret_cast<uintptr_t>(a->out) & 15) return TASP_EALIGN;
  const size_t need = tasp_chunk_attn_workspace_bytes(s, a);
  if (need > 0) {
    if (a->workspace == nullptr || a->workspace_bytes < need) return TASP_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(a->workspace) & (kAlign - 1)) return TASP_EALIGN;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  unsigned char* ws = static_cast<unsigned char*>(a->workspace);
  float* o_run = static_cast<float*>(a->out);           // fp32: the output itself is the running sum
  if (a->dtype == TASP_DTYPE_BF16) { o_run = reinterpret_cast<float*>(ws); ws += align_up(sh.o_bytes); }
  float* o_part = nullptr;
  float* lse_part = nullptr;
  if (!a->fuse_merge && !a->fuse_steps) {
    o_part = reinterpret_cast<float*>(ws); ws += align_up(sh.o_bytes);
    lse_part = reinterpret_cast<float*>(ws);
  }

  try {
    std::vector<tasp::QueryBlock> empty;
    if (a->fuse_steps) {
      AttnLaunch all{};
      {
        Scope sc(prof, Profiler::kOther);
        st = build_all_steps(s, a, reinterpret_cast<int32_t*>(ws), stream, &all);
        if (st != TASP_OK) return st;
      }
      all.o_dst = o_run; all.lse_dst = a->lse; all.merge = 0;
      {
        Scope sc(prof, Profiler::kAttn);
        if (launch_attn(all, a, stream) != hipSuccess) return TASP_EHIP;
      }
    }
    for (int step = 0; step < s->n && !a->fuse_steps; ++step) {
      AttnLaunch lp{};
      empty.clear();
      st = build_step(s, a, step, &lp, &empty);
      if (st != TASP_OK) return st;
      if (step == 0) {
        lp.o_dst = o_run; lp.lse_dst = a->lse; lp.merge = 0;
        {
          Scope sc(prof, Profiler::kAttn);
          if (launch_attn(lp, a, stream) != hipSuccess) return TASP_EHIP;
        }
        for (const auto& blk : empty)      // cannot happen with the placements of Sec. 3.2.3; kept for safety
          if (tasp::launch_fill_empty(o_run, a->lse, blk.local_row0, blk.rows, a->Hq, a->d, sh.B, sh.L, stream) !=
              hipSuccess)
            return TASP_EHIP;
      } else if (a->fuse_merge) {
        lp.o_dst = o_run; lp.lse_dst = a->lse; lp.merge = 1;
        Scope sc(prof, Profiler::kAttn);
        if (launch_attn(lp, a, stream) != hipSuccess) return TASP_EHIP;
      } else {
        lp.o_dst = o_part; lp.lse_dst = lse_part; lp.merge = 0;
        {
          Scope sc(prof, Profiler::kAttn);
          if (launch_attn(lp, a, stream) != hipSuccess) return TASP_EHIP;
        }
        // rows that saw no key at this step have nothing to fold in
        for (int t = 0; t < lp.n_tasks; ++t) {
          Scope sc(prof, Profiler::kMerge);
          if (tasp::launch_merge(o_run, a->lse, o_part, lse_part, lp.task[t].q_row0, lp.task[t].n_q, a->Hq, a->d,
                                 sh.B, sh.L, stream) != hipSuccess)
            return TASP_EHIP;
        }
      }
    }
    if (a->dtype == TASP_DTYPE_BF16) {
      Scope sc(prof, Profiler::kOther);
      if (tasp::launch_cast_bf16(o_run, a->out, sh.B * sh.L * a->Hq * a->d, stream) != hipSuccess) return TASP_EHIP;
    }
  } catch (...) {
    return TASP_ENOMEM;
  }
  return TASP_OK;
}

int tasp_chunk_attn(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream) {
  return run_chunk_attn(s, a, hip_stream, nullptr);
}

// Device address of `scratch` on the current device.  Every GPU holds its own copy of the array at
// its own address, so the address is asked for once per device, with that device current, and kept.
static int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (tasp::note_hip(hipGetDevice(&dev)) != hipSuccess) return TASP_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return TASP_EUNSUPPORTED_SHAPE;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (tasp::note_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) != hipSuccess || p == nullptr) return TASP_EHIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return TASP_OK;
}

int tasp_chunk_attn_static(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream) {
  if (s == nullptr || a == nullptr) return TASP_EINVAL;
  Shape sh;
  const int st = validate(s, a, &sh);
  if (st != TASP_OK) return st;
  // workspace_bytes() trusts its arguments; they have been validated above
  if (tasp_chunk_attn_workspace_bytes(s, a) > static_cast<size_t>(TASP_STATIC_SCRATCH_BYTES)) return TASP_EWORKSPACE;
  void* ws = nullptr;
  const int sp = static_scratch(&ws);
  if (sp != TASP_OK) return sp;
  tasp_attn_args b = *a;
  b.workspace = ws;
  b.workspace_bytes = TASP_STATIC_SCRATCH_BYTES;
  return run_chunk_attn(s, &b, hip_stream, nullptr);
}

size_t tasp_chunk_attn_bwd_workspace_bytes(const tasp_schedule_t* s, const tasp_attn_bwd_args* b) {
  if (s == nullptr || b == nullptr || b->S <= 0 || b->Hq <= 0 || b->d <= 0 || s->n <= 0 || b->batch < 0) return 0;
  const int64_t L = b->S / s->n;
  const size_t B = static_cast<size_t>(b->batch == 0 ? 1 : b->batch);
  if (b->dtype == TASP_DTYPE_FP32) return align_up(B * L * b->Hq * sizeof(float));   // delta; dq itself is the fp32 accumulator
  const size_t delta_bytes = align_up((B * L * b->Hq + 1) * sizeof(float));   // and the entry behind the last row
  const size_t table = b->fuse_steps ? align_up(kFusedTableBytes) : 0;    // segment lists of the single launch
  const size_t dq_bytes = align_up(B * L * b->Hq * b->d * sizeof(float));
  // step by step with grouped heads: partial dk and dv per query head of a step's L keys, fp32
  const size_t parts = (!b->fuse_steps && b->Hkv > 0 && b->Hq > b->Hkv) ? 2 * dq_bytes : 0;
  return dq_bytes + 2 * delta_bytes + table + parts;   // fp32 dq, delta, lse log2(e)
}

double tasp_chunk_attn_bwd_flops(const tasp_schedule_t* s, const tasp_attn_bwd_args* b) {
  if (s == nullptr || b == nullptr) return 0.0;
  const tasp_attn_args a = as_forward(b);
  return 2.5 * tasp_chunk_attn_flops(s, &a);
}

static int run_chunk_attn_bwd(const tasp_schedule_t* s, const tasp_attn_bwd_args* b, void* hip_stream, Profiler* prof) {
  Shape sh;
  tasp_attn_args a;
  int st = validate_bwd(s, b, &a, &sh);
  if (st != TASP_OK) return st;
  const size_t need = tasp_chunk_attn_bwd_workspace_bytes(s, b);
  if (b->workspace == nullptr || b->workspace_bytes < need) return TASP_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(b->workspace) & (kAlign - 1)) return TASP_EALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // With a second stream from the caller the dk/dv kernels run beside the dq kernels: fork after
  // delta is on its way, join before returning.  The profiled run keeps one stream (its events
  // bracket launches on `stream`).
  hipStream_t kv_stream = (b->aux_stream != nullptr && prof == nullptr) ? static_cast<hipStream_t>(b->aux_stream) : stream;
  struct Ev {
    hipEvent_t e = nullptr;
    ~Ev() { if (e) (void)hipEventDestroy(e); }
  } fork, join;
  const bool bf16 = b->dtype == TASP_DTYPE_BF16;
  float* dq_acc = bf16 ? static_cast<float*>(b->workspace) : static_cast<float*>(b->dq);
  float* delta = bf16 ? reinterpret_cast<float*>(static_cast<unsigned char*>(b->workspace) + align_up(sh.o_bytes))
                      : static_cast<float*>(b->workspace);
  const int64_t n_q_elems = static_cast<int64_t>(sh.B) * sh.L * b->Hq * b->d;
  const int64_t n_rows = static_cast<int64_t>(sh.B) * sh.L * b->Hq;
  // the dk/dv kernel addresses delta and lse2 with 32-bit byte offsets
  if (bf16 && n_rows >= (int64_t{1} << 30)) return TASP_EUNSUPPORTED_SHAPE;
  const size_t row_block = align_up(sh.lse_bytes + sizeof(float));
  float* lse2 = bf16 ? reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(delta) + row_block) : nullptr;
  unsigned char* after_rows = static_cast<unsigned char*>(b->workspace) + align_up(sh.o_bytes) + 2 * row_block;
  // partial dk / dv of a dk/dv launch split by query head (see launch_unit): room for L keys a launch
  float* part = (bf16 && !b->fuse_steps && b->Hq > b->Hkv) ? reinterpret_cast<float*>(after_rows) : nullptr;

  try {
    {
      Scope sc(prof, BwdSpans::kOther);
      const float scale = a.softmax_scale > 0.f ? a.softmax_scale : 1.0f / std::sqrt(static_cast<float>(a.d));   // as the launches below
      if ((bf16 ? tasp::launch_bwd_delta_bf16(b->out, b->dout, b->lse, delta, lse2, scale, n_rows, b->d, stream)
                : tasp::launch_bwd_delta_fp32(b->out, b->dout, delta, n_rows, b->d, stream)) != hipSuccess)
        return TASP_EHIP;
      if (tasp::launch_zero_f32(dq_acc, n_q_elems, stream) != hipSuccess) return TASP_EHIP;
    }
    if (kv_stream != stream) {
      if (tasp::note_hip(hipEventCreateWithFlags(&fork.e, hipEventDisableTiming)) != hipSuccess ||
          tasp::note_hip(hipEventCreateWithFlags(&join.e, hipEventDisableTiming)) != hipSuccess ||
          tasp::note_hip(hipEventRecord(fork.e, stream)) != hipSuccess ||
          tasp::note_hip(hipStreamWaitEvent(kv_stream, fork.e, 0)) != hipSuccess)
        return TASP_EHIP;
    }
    // One unit = one dq launch and one dk/dv launch: a step, or all steps at once.
    auto launch_unit = [&](const AttnLaunch& lp, std::vector<tasp::Segment>& ranges) -> int {
      tasp::BwdLaunch bp{};
      bp.q = b->q; bp.k = b->k; bp.v = b->v; bp.dout = b->dout; bp.lse = b->lse;
      if (bf16) { bp.ndelta = delta; bp.nlse = lse2; } else { bp.delta = delta; }
      bp.dq_acc = dq_acc; bp.dk = b->dk; bp.dv = b->dv;
      bp.Hq = lp.Hq; bp.Hkv = lp.Hkv; bp.causal = lp.causal; bp.scale = lp.scale; bp.batch = lp.batch;
      bp.q_bstride = lp.q_bstride; bp.kv_bstride = lp.kv_bstride; bp.lse_bstride = lp.lse_bstride;
      bp.n_tasks = lp.n_tasks;
      for (int t = 0; t < lp.n_tasks; ++t) { bp.task[t] = lp.task[t]; bp.seg_ext[t] = lp.seg_ext[t]; }
      bp.n_blk = tasp::n_query_blocks(b->mask_mode);
      for (int qb = 0; qb < bp.n_blk; ++qb) {
        tasp::QueryBlock blk;
        const int st2 = tasp::query_block(*s, b->S, b->mask_mode, qb, &blk);
        if (st2 != TASP_OK) return st2;
        bp.blk[qb] = {static_cast<int32_t>(blk.local_row0), static_cast<int32_t>(blk.rows), static_cast<int32_t>(blk.pos0)};
      }
      // The dk/dv kernel treats every key on its own, so the order of the ranges is free: by
      // position, which under the causal mask is by falling work (early keys are seen by more
      // queries), so that the workgroups with the most work start first.  Neighbours are joined.
      std::sort(ranges.begin(), ranges.end(),
                [](const tasp::Segment& x, const tasp::Segment& y) { return x.start < y.start; });
      size_t n = 0;
      for (size_t i = 0; i < ranges.size(); ++i) {
        if (n > 0 && ranges[n - 1].end == ranges[i].start) ranges[n - 1].end = ranges[i].end;
        else ranges[n++] = ranges[i];
      }
      if (n > static_cast<size_t>(tasp::kMaxSeg)) return TASP_EUNSUPPORTED_SHAPE;
      bp.n_rng = static_cast<int32_t>(n);
      int64_t vpos = 0;
      for (size_t i = 0; i < n; ++i) {
        bp.rng_start[i] = static_cast<int32_t>(ranges[i].start);
        bp.rng_vbeg[i] = static_cast<int32_t>(vpos);
        vpos += ranges[i].end - ranges[i].start;
      }
      bp.rng_vbeg[n] = static_cast<int32_t>(vpos);
      // A step's key tiles are few (S / N keys) and under the causal mask their work differs by
      // whole multiples (a tile is seen by both local half-chunks, by one, or by none), so the
      // launch ends with most CUs idle while a few finish a second tile.  Such a launch is cut
      // finer, one workgroup per key tile and query head; the partial sums are added up afterwards.
      // The finer launch costs a little where the coarse one is already even (partial sums written
      // and read back, more workgroup set-ups), so it is used where the estimate says it wins by more
      // than 4 %.
      bp.split_heads = 0;
      const int64_t wgs = tasp::bwd_dkv_workgroups(bp, b->d);
      const int slots = tasp::bwd_dkv_resident_workgroups(b->d);
      if (part != nullptr && vpos <= sh.L && wgs > 0 && wgs < 8 * static_cast<int64_t>(slots) &&
          dkv_makespan(bp, b->d, bp.Hq / bp.Hkv, slots) * 104 < dkv_makespan(bp, b->d, 1, slots) * 100) {
        bp.split_heads = 1;
        bp.part_dk = part;
        bp.part_dv = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(part) + align_up(sh.o_bytes));
      }
      {
        Scope sc(prof, BwdSpans::kDq);
        if ((bf16 ? tasp::launch_bwd_dq_bf16(bp, b->d, stream) : tasp::launch_bwd_dq_fp32(bp, b->d, stream)) != hipSuccess)
          return TASP_EHIP;
      }
      {
        Scope sc(prof, BwdSpans::kDkv);
        if ((bf16 ? tasp::launch_bwd_dkv_bf16(bp, b->d, kv_stream) : tasp::launch_bwd_dkv_fp32(bp, b->d, kv_stream)) !=
            hipSuccess)
          return TASP_EHIP;
      }
      if (bp.split_heads) {
        Scope sc(prof, BwdSpans::kOther);
        if (tasp::launch_bwd_dkv_reduce(bp, b->d, kv_stream) != hipSuccess) return TASP_EHIP;
      }
      return TASP_OK;
    };
    // All units; returns at the first failure, and the join below runs either way so that the
    // caller's second stream is never left forked (which would also break a stream capture).
    auto walk = [&]() -> int {
      std::vector<tasp::QueryBlock> empty;
      std::vector<tasp::Segment> ranges, step_ranges;
      if (b->fuse_steps) {
        AttnLaunch all{};
        int32_t* dev_table = reinterpret_cast<int32_t*>(after_rows);
        {
          Scope sc(prof, BwdSpans::kOther);
          st = build_all_steps(s, &a, dev_table, stream, &all);
          if (st != TASP_OK) return st;
        }
        for (int step = 0; step < s->n; ++step) {
          st = tasp::step_key_ranges(*s, b->S, b->mask_mode, b->order, step, &step_ranges);
          if (st != TASP_OK) return st;
          ranges.insert(ranges.end(), step_ranges.begin(), step_ranges.end());
        }
        st = launch_unit(all, ranges);
        if (st != TASP_OK) return st;
      }
      for (int step = 0; step < s->n && !b->fuse_steps; ++step) {
        AttnLaunch lp{};
        empty.clear();
        st = build_step(s, &a, step, &lp, &empty);
        if (st != TASP_OK) return st;
        st = tasp::step_key_ranges(*s, b->S, b->mask_mode, b->order, step, &ranges);
        if (st != TASP_OK) return st;
        st = launch_unit(lp, ranges);
        if (st != TASP_OK) return st;
      }
      return TASP_OK;
    };
    st = walk();
    if (kv_stream != stream) {
      if (tasp::note_hip(hipEventRecord(join.e, kv_stream)) != hipSuccess ||
          tasp::note_hip(hipStreamWaitEvent(stream, join.e, 0)) != hipSuccess)
        return st != TASP_OK ? st : TASP_EHIP;
    }
    if (st != TASP_OK) return st;
    if (bf16) {
      Scope sc(prof, BwdSpans::kOther);
      if (tasp::launch_cast_bf16(dq_acc, b->dq, n_q_elems, stream) != hipSuccess) return TASP_EHIP;
    }
  } catch (...) {
    return TASP_ENOMEM;
  }
  return TASP_OK;
}

int tasp_chunk_attn_bwd(const tasp_schedule_t* s, const tasp_attn_bwd_args* b, void* hip_stream) {
  return run_chunk_attn_bwd(s, b, hip_stream, nullptr);
}

int tasp_chunk_attn_bwd_profile(const tasp_schedule_t* s, const tasp_attn_bwd_args* b, void* hip_stream,
                                tasp_bwd_profile* out) {
  if (out == nullptr) return TASP_EINVAL;
  *out = tasp_bwd_profile{};
  try {
    Profiler prof;
    prof.stream = static_cast<hipStream_t>(hip_stream);
    const int st = run_chunk_attn_bwd(s, b, hip_stream, &prof);
    if (tasp::note_hip(hipStreamSynchronize(prof.stream)) != hipSuccess) return TASP_EHIP;
    if (st != TASP_OK) return st;
    if (prof.failed) return TASP_EHIP;
    for (const auto& sp : prof.spans) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, sp.beg, sp.end) != hipSuccess) return TASP_EHIP;
      if (sp.kind == BwdSpans::kDq) { out->dq_ms += ms; ++out->dq_launches; }
      else if (sp.kind == BwdSpans::kDkv) { out->dkv_ms += ms; ++out->dkv_launches; }
      else { out->other_ms += ms; ++out->other_launches; }
    }
  } catch (...) {
    return TASP_ENOMEM;
  }
  return TASP_OK;
}

int tasp_chunk_attn_profile(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream,
                            tasp_profile* out) {
  if (out == nullptr) return TASP_EINVAL;
  *out = tasp_profile{};
  try {
    Profiler prof;
    prof.stream = static_cast<hipStream_t>(hip_stream);
    const int st = run_chunk_attn(s, a, hip_stream, &prof);
    if (tasp::note_hip(hipStreamSynchronize(prof.stream)) != hipSuccess) return TASP_EHIP;
    if (st != TASP_OK) return st;
    if (prof.failed) return TASP_EHIP;
    for (const auto& sp : prof.spans) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, sp.beg, sp.end) != hipSuccess) return TASP_EHIP;
      if (sp.kind == Profiler::kAttn) { out->attn_ms += ms; ++out->attn_launches; }
      else if (sp.kind == Profiler::kMerge) { out->merge_ms += ms; ++out->merge_launches; }
      else { out->other_ms += ms; ++out->other_launches; }
    }
  } catch (...) {
    return TASP_ENOMEM;
  }
  return TASP_OK;
}

}  // extern "C"
