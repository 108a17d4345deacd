// Blockwise attention of one step of Algorithm 3 on gfx950: bf16 inputs, fp32 scores/softmax/output.
//
// The paper concatenates the N-1 sub-chunks of a step and calls a flash-attention library on the
// copy (Algorithm 3; Sec. 5.4 puts the cost of that copy at 1-5 % of the compute time).  Here the
// kernel walks the *virtual* concatenation instead: a workgroup owns 256 query rows of one head and
// streams 64-key tiles whose rows are gathered from the K/V segments of the step, so sub-chunk
// lengths that are no tile multiple cost nothing and nothing is copied.
//
// Per 32-row strip of queries:  S^T = K Q^T  and  O^T = V^T P^T  with v_mfma_f32_32x32x16_bf16.
// Computing the transposed products puts one query in one lane column, so the row max / row sum of
// the online softmax are in-lane reductions over 32 registers plus one exchange between the two
// lane halves, the rescale factor is a per-lane scalar, and the fp32 -> bf16 P tile is already in
// the B-operand layout of the second product.  K tiles are read from LDS with 16-byte reads, V
// tiles with the transposing LDS read (ds_read_b64_tr_b16); both tiles are XOR-swizzled in 16-byte
// units so that neither the fills nor the reads conflict on banks.
//
// The loop is software-pipelined by hand inside each wavefront: the second product of tile t and
// the scores of tile t+2 form one stream of matrix instructions that never drains (not at the
// barrier of a tile either), the softmax arithmetic of tiles t and t+1 is dealt out between them,
// operand fragments are read four ahead (two would do: the depth from 2 to 8 makes no measurable
// difference).  Matrix instructions and LDS reads are volatile assembly, so their order is the
// schedule.  K and V tiles arrive in two LDS rings of four tiles each through buffer loads that
// write LDS directly; the loop is unrolled four times, so that the ring stage of every tile is a
// constant and sits in the offset field of the LDS reads.
//
// What bounds it (measured with issue microbenchmarks on this chip): the vector issue port of a
// SIMD.  A matrix instruction occupies it for 12 cycles (and its own pipe for 32), a plain vector
// instruction for 4, an exponential for 8, and every KiB of LDS data returned to registers for
// about 4 more; per 64-key tile and wavefront that is 32 x 12 + 107 x 4 + 33 x 8 + 32 x 4 cycles,
// for two wavefronts more than the 2 048 cycles the matrix pipe needs.  So every vector instruction
// in the loop counts (hence the scalar bookkeeping of the loader, the stage offsets in the offset
// fields, the waits folded into the matrix instructions, the few branches), and beyond that the
// chip's power limit: with operands of ordinary statistics the clock falls as the pipes fill
// (about 1.7 GHz in this kernel against 2.4 GHz nominal), so cycles saved come back only in part.
//
// A wavefront owns NS strips.  NS = 1 (eight wavefronts, two per SIMD) is what the library
// launches.  NS = 2 (each LDS fragment feeds two matrix instructions, O^T and Q in AGPRs, one
// wavefront per SIMD) halves the LDS traffic and runs at a higher clock, but one wavefront issues a
// vector instruction only every five cycles and has to issue everything itself: 4 050 cycles per
// tile against 3 100, slower in time as well; kept as a template parameter.
#include <hip/hip_runtime.h>

#include <climits>

#include "gfx950.hpp"
#include "internal.hpp"

namespace tasp {
namespace {

constexpr int BN = 64;           // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleGap = 8.0f;   // the running max is only raised when it grew by more than 2^8
constexpr float kNegBig = -1.0e30f;

template <int D, int NS_, int NW_>
struct Cfg {
  static constexpr int NS = NS_;                      // 32-row query strips per wavefront
  static constexpr int NWAVES = NW_;                  // 8: two wavefronts per SIMD, 12: three (fits at D = 64), 4 with NS = 2: one
  static constexpr int NTHREADS = 64 * NWAVES;
  static constexpr int BM = 32 * NS * NWAVES;         // query rows per workgroup (256)
  static constexpr int UNITS = D / 8;                 // 16-byte units per row
  static constexpr int RPP = NTHREADS / UNITS < BN ? NTHREADS / UNITS : BN;   // rows filled per pass
  static constexpr int LOADERS = RPP * UNITS;         // threads that fetch tiles (the first LOADERS / 64 wavefronts)
  static constexpr int PASSES = BN / RPP;
  static constexpr int ROWS_PER_LINE = 16 / UNITS;    // rows per 256-byte bank line (1 or 2)
  static constexpr int TILE_BYTES = BN * D * 2;
  static constexpr int STAGES = 4;
  static constexpr int SMEM = STAGES * 2 * TILE_BYTES;   // ring of K tiles, then ring of V tiles
  static constexpr int V_RING = STAGES * TILE_BYTES;     // where the V ring starts
  static_assert(V_RING <= 65536, "stage and fragment offsets of an LDS read go into its 16-bit offset field");
  __device__ static int swz_k(int row, int unit) { return unit ^ ((row / ROWS_PER_LINE) % UNITS); }
  __device__ static int swz_v(int row, int unit) { return unit ^ (4 * ((row / ROWS_PER_LINE) % (UNITS / 4))); }
};

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// maxima as assembly: the inputs come out of matrix instructions the compiler cannot see, and it
// would otherwise quiet every one of them first
__device__ __forceinline__ float max2(float a, float b) { float r; asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ float max3(float a, float b, float c) { float r; asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c)); return r; }

// Tile fetches use the direct global->LDS load without a compiler-level fence: the wait for it is
// placed by hand (s_waitcnt vmcnt before the barrier that publishes the tile), no other vector
// memory instruction is in flight while these are, the stage it fills is not read before the next
// barrier, and barriers and waits are ordered against volatile assembly.
__device__ inline void dma16(const u32x4& rsrc, unsigned soff, unsigned off, unsigned char* lds_base) {
  buffer_to_lds_16(rsrc, soff, off, lds_base);
}

// LDS operand reads whose wait is placed by hand.  A read is volatile assembly (issued in program
// order), and the fragment reaches its matrix instruction only behind a wait until at most N
// younger LDS instructions are outstanding (LDS instructions of a wavefront complete in order, so
// extra ones the compiler adds only make a wait stricter).  In the loop that wait is part of the
// matrix instruction's own asm statement (TASP_MFMA_ASM); lds_wait is the stand-alone form.
template <int IMM>
__device__ __forceinline__ void lds_read_b128(u32x4& d, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(IMM));
}
template <int IMM>
__device__ __forceinline__ void lds_read_tr_b64(u32x2& d, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(IMM));
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x4& f) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f) : "n"(N));
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x2& a, u32x2& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}

// Matrix instructions as volatile assembly: they stay in program order, which is the schedule, and
// the register classes are fixed: score tiles in VGPRs (the softmax reads them), O^T and the Q
// fragments in AGPRs.  The compiler does not know these are matrix instructions, so the wait states
// it would insert are placed by hand (the fence_* helpers):
//   matrix result -> vector ALU / accvgpr read: 12 wait states;  vector ALU result -> matrix operand: 2.
// Dependent matrix instructions on the same accumulator need none.
// ACC: O^T and the Q fragments live in AGPRs (needed when a wave owns two strips; with one strip
// everything fits the 256 VGPRs of a wave that shares its SIMD, and using any AGPR would make the
// compiler split that budget in half).
// W >= 0: the instruction's fragment `a` comes from LDS reads in flight, and the wait for it (at most
// W younger LDS instructions outstanding) sits in the same asm statement: a wait in a statement of
// its own that names the fragment makes the compiler put a wait state between the two (it has to
// assume that any asm statement forwards its result like a sub-dword write).  W < 0: no wait.
#define TASP_MFMA_ASM(W, ...)                                                                   \
  do {                                                                                          \
    if constexpr ((W) >= 0) asm volatile("s_waitcnt lgkmcnt(%3)\n\t" __VA_ARGS__, "n"((W) < 0 ? 0 : (W))); \
    else asm volatile(__VA_ARGS__, "n"(0));                                                     \
  } while (0)
template <bool ACC, int W = -1>
__device__ __forceinline__ void mfma_s_first(f32x16& d, const u32x4& a, const u32x4& b) {
  if constexpr (ACC) TASP_MFMA_ASM(W, "v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
  else TASP_MFMA_ASM(W, "v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
}
template <bool ACC, int W = -1>
__device__ __forceinline__ void mfma_s(f32x16& d, const u32x4& a, const u32x4& b) {
  if constexpr (ACC) TASP_MFMA_ASM(W, "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
  else TASP_MFMA_ASM(W, "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
template <bool ACC, int W = -1>
__device__ __forceinline__ void mfma_o(f32x16& d, const u32x4& a, const u32x4& b) {
  if constexpr (ACC) TASP_MFMA_ASM(W, "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
  else TASP_MFMA_ASM(W, "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
// score tile: readable by the vector ALU after this point (placed at least one matrix instruction after the last one that wrote it)
__device__ __forceinline__ void fence_s(f32x16& a, f32x16& b) { asm volatile("s_nop 15" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void fence_s_next(f32x16& a, f32x16& b) { asm volatile("" : "+v"(a), "+v"(b)); }
// P fragment: written by the vector ALU, read by matrix instructions after this point
__device__ __forceinline__ void fence_p(u32x4& f) { asm volatile("s_nop 1" : "+v"(f)); }
// O^T accumulator: readable / writable by the vector ALU after this point
template <bool ACC>
__device__ __forceinline__ void fence_o_first(f32x16& a) {
  if constexpr (ACC) asm volatile("s_nop 15\n\ts_nop 3" : "+a"(a));
  else asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a));
}
template <bool ACC>
__device__ __forceinline__ void fence_o_next(f32x16& a) {
  if constexpr (ACC) asm volatile("" : "+a"(a));
  else asm volatile("" : "+v"(a));
}
// O^T accumulator written by the vector ALU, read by matrix instructions after this point
template <bool ACC>
__device__ __forceinline__ void fence_o_written(f32x16& a) {
  if constexpr (ACC) asm volatile("s_nop 1" : "+a"(a));
  else asm volatile("s_nop 1" : "+v"(a));
}

template <int D, int NS, int NW, bool PERSIST>
__global__ __launch_bounds__(64 * NW, NW / 4) void attn_bf16_kernel(const AttnLaunch p) {
  using C = Cfg<D, NS, NW>;
  constexpr int BM = C::BM;
  constexpr int KS = D / 16;     // contraction steps of K Q^T
  constexpr int DB = D / 32;     // 32-row blocks of O^T
  constexpr bool ACC = NS > 1;

  __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];   // four K tiles, then four V tiles
  __shared__ __attribute__((aligned(16))) int s_tok[C::STAGES][BN];   // global position of every key row of a tile (INT_MAX: none)
  // Effective segments: the segments are disjoint ranges of the sequence, so at most one of them
  // holds the first position of the query tile and is split in two; hence kMaxSegAll + 2 entries.
  __shared__ int e_vbeg[kMaxSegAll + 2];   // start in the virtual concatenation
  __shared__ int e_goff[kMaxSegAll + 2];   //   global position minus virtual position
  __shared__ int e_diag[kMaxSegAll + 2];   //   straddles the diagonal of this query tile
  __shared__ int e_n;
  __shared__ int m_lo[kMaxSegAll + 2];     // runs of tiles that need the element-wise mask (sorted, the
  __shared__ int m_hi[kMaxSegAll + 2];     //   last run is open-ended: m_hi = INT_MAX)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int h = lane >> 5;       // lane half
  const int lq = lane & 31;      // query column inside a strip

  // ---- which (KV head, task, query tile, query head) this workgroup owns.  Workgroups are dealt
  // round-robin to the 8 XCDs; the index is remapped so that each XCD gets a contiguous run of work
  // ordered KV-head-major: the workgroups of one XCD then stream the same K/V through its L2 (and
  // XCDs that have to share KV heads deal the items of those heads among them: xcd_balanced).
  const int G = p.Hq / p.Hkv;
  const int tiles0 = (p.task[0].n_q + BM - 1) / BM;
  const int tiles1 = p.n_tasks > 1 ? (p.task[1].n_q + BM - 1) / BM : 0;
  const int per_g = (tiles0 + tiles1) * G;
  const int per_b = per_g * p.Hkv;                            // work items of one sequence of the batch
  // With PERSIST there is one workgroup per CU and it takes several work items in turn, which
  // saves the 4 us a CU idles between two workgroups.  The outer loop costs registers, so this pays
  // only where there are registers to spare and the items are short: d = 64, all steps in one launch.
  for (int round = 0; PERSIST || round == 0; ++round) {
  const int w_all = PERSIST ? persistent_item(blockIdx.x, gridDim.x, p.n_items, round) : xcd_balanced(blockIdx.x, p.batch * p.Hkv, per_g);
  if (w_all < 0) break;
  const int bi = w_all / per_b;
  const int w = w_all - bi * per_b;
  const int g = w / per_g;
  int rem = w - g * per_g;
  const int tsk = rem >= tiles0 * G ? 1 : 0;
  if (tsk) rem -= tiles0 * G;
  // under the causal mask the later query tiles of a block see more keys: they start first
  const int tile_q = p.causal ? (tsk ? tiles1 : tiles0) - 1 - rem / G : rem / G;
  const int hq = g * G + rem % G;
  const AttnTask& T = p.task[tsk];
  const int q_tile_row0 = tile_q * BM;                        // relative to the task
  const int q_rows_here = min(BM, T.n_q - q_tile_row0);
  const int qa = T.q_pos0 + q_tile_row0;                      // first and last position of the tile
  const int qb = qa + q_rows_here - 1;

  // ---- Q fragments (B operand of K Q^T), strip s: lane holds query 32 s + lq, d = 16 ks + 8 h .. +8.
  // Issued first: their way from memory overlaps the construction of the segment list below.
  int my_q[NS], q_pos[NS];
  bool q_valid[NS];
  u32x4 qf[NS][KS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    my_q[s] = q_tile_row0 + wave * (32 * NS) + 32 * s + lq;          // row inside the task
    q_valid[s] = my_q[s] < T.n_q;
    const int64_t q_row = T.q_row0 + (q_valid[s] ? my_q[s] : T.n_q - 1);
    const __bf16* src = static_cast<const __bf16*>(p.q) + bi * p.q_bstride + (q_row * p.Hq + hq) * D + 8 * h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[s][ks] = *reinterpret_cast<const u32x4*>(src + 16 * ks);
    q_pos[s] = p.causal ? T.q_pos0 + my_q[s] : INT_MAX - 1;
  }
  // ---- effective segment list of this query tile: drop what the causal mask hides from every
  // row, split the rest into a part every row sees and a part that straddles the diagonal.
  // The list - from the descriptor, or in single-launch mode from device memory - is staged in
  // the (still unused) tile ring first.
  const int32_t* seg_ext = p.seg_ext[tsk];
  int* seg_raw = reinterpret_cast<int*>(smem);
  if (seg_ext != nullptr) {
    for (int i = tid; i < 2 * T.n_seg; i += C::NTHREADS) seg_raw[i] = seg_ext[i];
  } else if (tid < T.n_seg) {
    seg_raw[2 * tid] = T.seg_start[tid];
    seg_raw[2 * tid + 1] = T.seg_end[tid];
  }
  __syncthreads();
  // The first wavefront builds the list, 64 segments per round: every lane classifies one segment
  // on its own; only the positions in the list and in the virtual concatenation are running sums
  // (wavefront scans).  The tile ranges of the diagonal parts go to m_lo / m_hi first and are
  // merged into runs in place by one lane.
  if (wave == 0) {
    int n_base = 0, v_base = 0, d_base = 0;      // entries, keys and diagonal entries so far (uniform)
    for (int s0 = 0; s0 < T.n_seg; s0 += 64) {
      const int s = s0 + lane;
      int a = 0, len_f = 0, len_d = 0, start_d = 0;
      if (s < T.n_seg) {
        a = seg_raw[2 * s];
        const int b = seg_raw[2 * s + 1];
        if (!p.causal) {
          len_f = b - a;
        } else if (a <= qb) {
          const int b_vis = min(b, qb + 1);
          const int full_end = min(b_vis, qa + 1);        // keys before it are seen by every row of the tile
          len_f = max(0, full_end - a);
          start_d = max(a, full_end);
          len_d = max(0, b_vis - start_d);
        }
      }
      const int cnt = (len_f > 0 ? 1 : 0) + (len_d > 0 ? 1 : 0), len = len_f + len_d, dg = len_d > 0 ? 1 : 0;
      int sc = cnt, sl = len, sd = dg;                      // inclusive scans
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t1 = __shfl_up(sc, o), t2 = __shfl_up(sl, o), t3 = __shfl_up(sd, o);
        if (lane >= o) { sc += t1; sl += t2; sd += t3; }
      }
      int idx = n_base + sc - cnt, vpos = v_base + sl - len;
      const int didx = d_base + sd - dg;
      if (len_f > 0) { e_vbeg[idx] = vpos; e_goff[idx] = a - vpos; e_diag[idx] = 0; ++idx; vpos += len_f; }
      if (len_d > 0) {
        e_vbeg[idx] = vpos; e_goff[idx] = start_d - vpos; e_diag[idx] = 1;
        m_lo[didx] = vpos / BN; m_hi[didx] = (vpos + len_d - 1) / BN;
      }
      n_base += __shfl(sc, 63); v_base += __shfl(sl, 63); d_base += __shfl(sd, 63);
    }
    if (lane == 0) {
      e_vbeg[n_base] = v_base;
      e_n = n_base;
      // runs of tiles that touch a diagonal part, and everything from the first tile that runs past the last key
      int mn = 0, cur_lo = -1, cur_hi = -1;
      for (int k = 0; k < d_base; ++k) {
        const int lo = m_lo[k], hi = m_hi[k];
        if (cur_lo >= 0 && lo <= cur_hi) { cur_hi = max(cur_hi, hi); continue; }
        if (cur_lo >= 0) { m_lo[mn] = cur_lo; m_hi[mn] = cur_hi; ++mn; }    // mn <= k: entry k has been read
        cur_lo = lo; cur_hi = hi;
      }
      const int tail = v_base / BN;
      if (cur_lo >= 0 && tail <= cur_hi) {
        m_lo[mn] = cur_lo; m_hi[mn] = INT_MAX;
      } else {
        if (cur_lo >= 0) { m_lo[mn] = cur_lo; m_hi[mn] = cur_hi; ++mn; }
        m_lo[mn] = tail; m_hi[mn] = INT_MAX;
      }
    }
  }
  __syncthreads();
  const int n_eff = e_n;
  const int total_keys = e_vbeg[n_eff];
  const int n_tiles = (total_keys + BN - 1) / BN;

  // Land the Q fragments now (vmcnt(0)): the waits for the tile fetches below count vector memory
  // instructions and assume that nothing else is in flight.
  __builtin_amdgcn_s_waitcnt(0x0F70);

  // ---- loader: this thread fills rows fr + RPP*i, unit fu of every K and V tile.  Byte offsets
  // into K and V fit 32 bits (checked on the host).
  const int fr = tid / C::UNITS, fu = tid % C::UNITS;
  const unsigned row_bytes = static_cast<unsigned>(p.Hkv) * D * 2;
  // Row bookkeeping of the loader.  One wavefront-load covers RW consecutive rows of a tile, and as
  // long as these are RW consecutive keys of one effective segment, the address of a lane is a
  // wavefront-uniform base plus a per-lane constant.  So on the common path everything is scalar:
  // per pass the wavefront follows the first of its RW rows through the virtual concatenation
  // (w_tok = its global position; w_left = keys from it to the end of its segment; w_seg = its
  // segment; k_off = byte offset of that key's row), from one tile to the next all of these move 64
  // keys on, the loads take k_off as their scalar offset and their lane offsets (lane_k, lane_v)
  // never change.  Only when fewer than RW keys are left in the segment, or the
  // tile runs past the last key (one tile in about ten with sub-chunks of a thousand keys) every
  // lane searches the segment list for its own row and gets an offset of its own (base offset 0).
  // A vector instruction costs the SIMD's issue port as much as a third of a matrix instruction,
  // and the port is what bounds this kernel.
  constexpr int RW = 64 / C::UNITS;
  const int r_lane = lane / C::UNITS;
  const unsigned k_col = C::swz_k(fr, fu) * 16, v_col = C::swz_v(fr, fu) * 16;    // byte column this lane reads
  static_assert(C::RPP % 16 == 0, "the swizzle of a thread's rows must not depend on the pass");
  const unsigned lane_k_const = static_cast<unsigned>(r_lane) * row_bytes + k_col;
  int w_tok[C::PASSES], w_left[C::PASSES], w_seg[C::PASSES];
  unsigned k_off[C::PASSES], v_off[C::PASSES];       // scalar: byte offset of the pass's first row, tile u / tile u-1
  unsigned lane_k[C::PASSES], lane_v[C::PASSES];     // per lane: added to it
#pragma unroll
  for (int i = 0; i < C::PASSES; ++i) {
    w_tok[i] = 0; w_left[i] = 0; w_seg[i] = 0; k_off[i] = 0; v_off[i] = 0;
    lane_k[i] = lane_k_const; lane_v[i] = lane_k_const + (v_col - k_col);
  }
  int tokk[C::PASSES];           // global position of this lane's row of the tile being fetched
  // The lane offsets differ from their constants while a tile with a searched pass is on its way:
  // its K loads (this round), its V loads (next round), and back (the round after).  hist = which
  // of the last two tiles had one; slow_below = RW, or INT_MAX while hist is not 0.
  int hist = 0, slow_below = RW;
  // every lane finds its own row of tile t (pass i); the wavefront's state is taken from its first lane
  auto locate_slow = [&](int i, int t) __attribute__((always_inline)) {
    const int v = t * BN + fr + C::RPP * i;
    int j = w_seg[i], left;                                   // rows only move forward
    while (j < n_eff && v >= e_vbeg[j + 1]) ++j;
    if (j < n_eff) { tokk[i] = v + e_goff[j]; left = e_vbeg[j + 1] - v; }
    else { tokk[i] = INT_MAX; left = 0; }                     // past the last key: searched again next time
    w_tok[i] = __builtin_amdgcn_readfirstlane(tokk[i]);
    w_left[i] = __builtin_amdgcn_readfirstlane(left);
    w_seg[i] = __builtin_amdgcn_readfirstlane(j);
  };
  // rows of tile t; must be called for t = 0, 1, 2, ... in this order
  auto locate = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < C::PASSES; ++i) {
      v_off[i] = k_off[i];                                    // V of the tile before goes out this round
      w_left[i] -= BN;                                        // tile 0: from 0, i.e. search
      w_tok[i] += BN;
      k_off[i] += BN * row_bytes;
      tokk[i] = w_tok[i] + r_lane;
      // The new values are pinned to scalar registers here.  Left alone, the compiler moves these
      // additions behind the branch below (the other arm overwrites them), which leaves an undefined
      // input at the join, and it resolves that by keeping the whole chain in vector registers.
      asm volatile("" : "+s"(k_off[i]), "+s"(w_tok[i]), "+s"(w_left[i]));
    }
    int least = w_left[0];                                    // (a three-way minimum would become a vector instruction)
#pragma unroll
    for (int i = 1; i < C::PASSES; ++i) least = min(least, w_left[i]);
    if (__builtin_expect(least < slow_below, 0)) {
      int slow = 0;
#pragma unroll
      for (int i = 0; i < C::PASSES; ++i) {
        lane_v[i] = lane_k[i] + (v_col - k_col);             // unsigned wrap-around is exact
        lane_k[i] = lane_k_const;
        k_off[i] = static_cast<unsigned>(w_tok[i]) * row_bytes;
        asm volatile("" : "+s"(k_off[i]));                    // (pinned, as above)
        if (w_left[i] < RW) {
          locate_slow(i, t);
          // rows past the end fetch key 0 and are masked; both factors are below 2^24 (host check)
          lane_k[i] = __umul24(tokk[i] == INT_MAX ? 0u : static_cast<unsigned>(tokk[i]), row_bytes) + k_col;
          k_off[i] = 0;
          slow = 1;
        }
      }
      hist = ((hist << 1) | slow) & 3;
      slow_below = hist != 0 ? INT_MAX : RW;
    }
  };
  // Tiles go straight into the rings (global_load_lds: no registers, no LDS write instructions).
  // A wavefront's 64 lanes fill 1 KiB of consecutive LDS; the XOR swizzle of the tile layout is
  // applied on the source side: the lane that owns LDS slot (row, unit) reads the 16 bytes of column
  // swz(row, unit) of that row.
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // wavefront-uniform, and known at compile time when every wavefront fetches (a branch costs a
  // wavefront 20-40 cycles even when it is not taken)
  const bool is_loader = C::LOADERS == C::NTHREADS || wave_u < C::LOADERS / 64;
  const unsigned char* Kg = static_cast<const unsigned char*>(p.k) + (bi * p.kv_bstride + static_cast<int64_t>(g) * D) * 2;   // this sequence and KV head, uniform
  const unsigned char* Vg = static_cast<const unsigned char*>(p.v) + (bi * p.kv_bstride + static_cast<int64_t>(g) * D) * 2;
  const u32x4 k_buf = raw_buffer(Kg), v_buf = raw_buffer(Vg);
  // Round u of the fetch brings K(u) into stage u % 4 of the K ring and V(u-1) into stage (u-1) % 4
  // of the V ring (the main loop says why the two halves of a tile travel a round apart); 2*PASSES
  // loads per thread.  The path from L2 into LDS takes roughly 25 cycles per wavefront-load and the
  // issuing wave stalls once its queue is full, so the loads are not issued in one burst:
  // fetch_begin(u) does the bookkeeping of tile u, fetch_piece(j) issues load j (even: K(u), pass
  // j/2; odd: V(u-1)), and the loop drops the pieces between its matrix instructions.
  unsigned char* fetch_dst_k = smem;
  unsigned char* fetch_dst_v = smem;
  auto fetch_begin = [&](int u, auto us_) __attribute__((always_inline)) {      // us_ = u % 4 at compile time
    constexpr int US = decltype(us_)::value;
    if (!is_loader) return;
    locate(u);
    fetch_dst_k = smem + US * C::TILE_BYTES + wave_u * 1024;
    fetch_dst_v = smem + C::V_RING + ((US + 3) & 3) * C::TILE_BYTES + wave_u * 1024;
#pragma unroll
    for (int i = 0; i < C::PASSES; ++i) s_tok[US][fr + C::RPP * i] = tokk[i];    // the UNITS lanes of a row write the same value
  };
  auto fetch_piece = [&](int j, bool with_v = true) __attribute__((always_inline)) {
    const int i = j >> 1;
    if (!is_loader) return;
    if (j & 1) {
      if (with_v) dma16(v_buf, v_off[i], lane_v[i], fetch_dst_v + i * C::LOADERS * 16);
    } else {
      dma16(k_buf, k_off[i], lane_k[i], fetch_dst_k + i * C::LOADERS * 16);
    }
  };
  auto fetch_round = [&](int u, auto us_, bool with_v) __attribute__((always_inline)) {
    fetch_begin(u, us_);
#pragma unroll
    for (int j = 0; j < 2 * C::PASSES; ++j) fetch_piece(j, with_v);
  };
  // wait until at most `newest` of this wave's tile fetches (each 2*PASSES loads) are still in flight
  auto wait_fetches = [&](auto newest) __attribute__((always_inline)) {
    constexpr int N = decltype(newest)::value * 2 * C::PASSES;
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  };

  constexpr std::integral_constant<int, 0> stage0{};
  constexpr std::integral_constant<int, 1> stage1{};
  constexpr std::integral_constant<int, 2> stage2{};
  constexpr std::integral_constant<int, 3> stage3{};

  // ---- per-lane LDS read addresses, stage 0 (loop invariant)
  const unsigned smem_lds = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)smem));
  unsigned kadr[KS];  // K: row lq (+32 kb), unit 2 ks + h
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kadr[ks] = smem_lds + (lq * C::UNITS + C::swz_k(lq, 2 * ks + h)) * 16;
  // V^T through the transposing read: 16-lane group a = lane/16 serves d columns 16 (a%2) .. +16 of
  // a 32-wide block for lane half h = a/2; lane jj of the group points at key 4 h + jj/4, 4 d values.
  const int ga = lane >> 4, jj = lane & 15;
  const int vrow = 4 * (ga >> 1) + (jj >> 2);                 // key row inside a 16-key block (+8 second read)
  unsigned vadr[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    const int unit = 4 * db + 2 * (ga & 1) + ((jj & 3) >> 1);
    vadr[db] = smem_lds + C::V_RING + (vrow * C::UNITS + C::swz_v(vrow, unit)) * 16 + 8 * (jj & 1);
  }

  // ---- running state, per strip
  f32x16 o[NS][DB];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[s][db][i] = 0.f;
  // Running max in the exp2 domain (scaled scores times log2 e) and this lane's share of the
  // running sum.  The sum is kept in two levels - the last (up to) 64 tiles in l_lo, everything
  // before in l_run - because a single fp32 accumulator that already holds a few large terms
  // swallows the many small ones that follow (each below half an ulp of it): with a million keys
  // and outlier scores that alone costs up to 1e-3 in lse.  The sum of 64 tiles is large enough to
  // register, and a large term sits in l_lo for 64 tiles at most.
  // The second product sees P rounded to bf16 while l adds up the fp32 values, so a row that a few
  // keys dominate would come out scaled by the rounding error of their probabilities: up to 2^-9 of
  // its value, 0.01 where |v| reaches 5, on top of the final rounding of the output.  r_fix collects,
  // per 64-key tile, what the rounding added to the largest probability each lane holds; the output
  // is divided by l + r_fix, which cancels the error of every dominant key to first order (keys that
  // dominate from the same 32 scores of a lane share one correction).  Summing all rounded
  // probabilities would be exact, but v_dot2c_f32_bf16 is a half-rate instruction: 10 % of the
  // vector port.  lse comes from l alone.
  float m_run[NS], m_raise[NS], l_run[NS], l_lo[NS], r_fix[NS];     // m_raise = m_run + the gap
#pragma unroll
  for (int s = 0; s < NS; ++s) { m_run[s] = kNegBig; m_raise[s] = kNegBig; l_run[s] = 0.f; l_lo[s] = 0.f; r_fix[s] = 0.f; }
  const float c = p.scale * kLog2e;
  auto fence_o = [&]() __attribute__((always_inline)) {
    fence_o_first<ACC>(o[0][0]);
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        if (s + db > 0) fence_o_next<ACC>(o[s][db]);
  };

  // a score tile becomes readable by the vector ALU
  auto fence_scores = [&](f32x16 (&S)[NS][2]) __attribute__((always_inline)) {
    fence_s(S[0][0], S[0][1]);
#pragma unroll
    for (int s = 1; s < NS; ++s) fence_s_next(S[s][0], S[s][1]);
  };

  // element-wise mask of the scores of tile t, only for tiles that touch the diagonal or run past the last key
  int m_idx = 0;
  int m_cur_lo = __builtin_amdgcn_readfirstlane(m_lo[0]), m_cur_hi = __builtin_amdgcn_readfirstlane(m_hi[0]);
  auto mask = [&](auto ts_, int t, f32x16 (&S)[NS][2]) __attribute__((always_inline)) {
    if (__builtin_expect(t < m_cur_lo, 1)) return;     // one compare on the common path (m_cur_lo <= m_cur_hi)
    while (t > m_cur_hi) {     // t only grows; the last run never ends
      ++m_idx;
      m_cur_lo = __builtin_amdgcn_readfirstlane(m_lo[m_idx]);
      m_cur_hi = __builtin_amdgcn_readfirstlane(m_hi[m_idx]);
    }
    if (t >= m_cur_lo) {
      constexpr int stage = decltype(ts_)::value;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const i32x4 tk = *reinterpret_cast<const i32x4*>(&s_tok[stage][32 * kb + 8 * i4 + 4 * h]);
#pragma unroll
          for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (tk[e] > q_pos[s]) S[s][kb][4 * i4 + e] = -__builtin_inff();
        }
    }
  };
  // row maximum of a score tile, in 16 steps per strip
  float mx[NS];
  auto max_step = [&](auto ii, f32x16 (&S)[NS][2]) __attribute__((always_inline)) {
    constexpr int I = decltype(ii)::value;       // strip I % NS, scores 2 (I / NS), 2 (I / NS) + 1 of the 32 a lane holds
    constexpr int s = I % NS, kb = I / NS / 8, e = 2 * ((I / NS) % 8);
    if constexpr (I / NS == 0) mx[s] = max2(S[s][kb][e], S[s][kb][e + 1]);
    else mx[s] = max3(mx[s], S[s][kb][e], S[s][kb][e + 1]);
  };
  // after the 16 steps: fold the lane halves, raise the running max lazily (only when it grew by more
  // than 2^8) and rescale what has been accumulated; the second product of the tile before must be complete
  // (a lane tests the 32 scores it holds itself: a row has grown iff one of its two lanes has, and
  // the exchange between the lane halves is needed only then)
  auto raise_max = [&]() __attribute__((always_inline)) {
    bool grew = false;
#pragma unroll
    for (int s = 0; s < NS; ++s) grew |= mx[s] * c > m_raise[s];
    if (__builtin_amdgcn_ballot_w64(grew) != 0) {
      fence_o();
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const unsigned mu = __builtin_bit_cast(unsigned, mx[s]);
        const u32x2 sw = __builtin_amdgcn_permlane32_swap(mu, mu, false, false);   // the other 16 keys of a block sit 32 lanes away
        const float m2 = max2(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1]));
        const float m_cand = max2(m_run[s], m2 * c);
        const float alpha = fast_exp2(m_run[s] - m_cand);
        m_run[s] = m_cand;
        m_raise[s] = m_cand + kRescaleGap;
        l_run[s] *= alpha;
        l_lo[s] *= alpha;
        r_fix[s] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
          for (int i = 0; i < 16; ++i) o[s][db][i] *= alpha;
          fence_o_written<ACC>(o[s][db]);
        }
      }
    }
  };
  // P = exp2(S c - m) for two neighbouring scores of a lane, packed to bf16 into the B-operand
  // fragment of its 16-key group.  Pair index: group g = PI / 8 (kb = g / 2, j = g % 2), strip (PI % 8) / 4.
  u32x4 pf[NS][4];
  // The exponential of an element is issued one element before its result is used (sum, packing):
  // a transcendental takes longer than the instruction behind it would wait.
  float x_late = 0.f, x_later = 0.f;   // exp of element EI-1, EI-2
  auto use_exp = [&](auto ei) __attribute__((always_inline)) {      // consume element EI, whose exp is x_late (x_later holds EI-1)
    constexpr int EI = decltype(ei)::value;
    constexpr int gg = EI / (8 * NS), s = (EI % (8 * NS)) / 8, e = EI % 8;
    l_lo[s] += x_late;
    asm volatile("" : "+v"(l_lo[s]));            // keeps the addition here instead of in a later block
    if constexpr (e % 2 == 1) {
      const bf16x2 pk = {static_cast<__bf16>(x_later), static_cast<__bf16>(x_late)};
      pf[s][gg][e / 2] = __builtin_bit_cast(unsigned, pk);
    }
  };
  constexpr int NE_ = 32 * NS;
  auto exp_one = [&](auto ei, f32x16 (&S)[NS][2]) __attribute__((always_inline)) {
    constexpr int EI = decltype(ei)::value;      // element: group EI / (8 NS) (kb = g / 2, j = g % 2), strip (EI % (8 NS)) / 8, score EI % 8 of the group
    constexpr int gg = EI / (8 * NS), s = (EI % (8 * NS)) / 8, e = EI % 8, kb = gg / 2, j = gg % 2;
    const float x = fast_exp2(__builtin_fmaf(S[s][kb][8 * j + e], c, -m_run[s]));
    if constexpr (EI > 0) use_exp(std::integral_constant<int, EI - 1>{});
    x_later = x_late;
    x_late = x;
    if constexpr (EI == NE_ - 1) use_exp(ei);    // the last one is needed right away
  };

  // ---- the matrix instructions of a loop body as one stream of operand fragments: fragments
  // 0..NKF-1 are K (scores of tile t+1, contraction step f/2, key block f%2), the rest V^T (second
  // product of tile t, 16-key group and 32-row block of O^T); each feeds the two strips.  The reads
  // of fragment f+PD are issued when fragment f has been consumed.
  constexpr int NKF = 2 * KS, NVF = 4 * DB, NF = NKF + NVF;
  constexpr int NKM = NS * NKF, NVM = NS * NVF;        // matrix instructions per phase
  constexpr int PD = 4;
  static_assert(NKF >= PD && NVF >= PD, "");
  u32x4 fk[PD];            // K fragments in flight (ring slot = fragment % PD)
  u32x2 fl[PD], fh[PD];    // V^T fragments in flight, low and high half
  // (sk, sv: ring stages of the K and the V tile, compile-time, so they go into the offset field)
  auto issue = [&](auto ff, auto sk_, auto sv_) __attribute__((always_inline)) {
    constexpr int F = decltype(ff)::value, slot = F % PD;
    constexpr int SK = decltype(sk_)::value * C::TILE_BYTES, SV = decltype(sv_)::value * C::TILE_BYTES;
    if constexpr (F < NKF) {
      constexpr int ks = F / 2, kb = F % 2;
      lds_read_b128<kb * 32 * D * 2 + SK>(fk[slot], kadr[ks]);
    } else {
      constexpr int gg = (F - NKF) / DB, db = (F - NKF) % DB;
      lds_read_tr_b64<gg * 16 * D * 2 + SV>(fl[slot], vadr[db]);
      lds_read_tr_b64<gg * 16 * D * 2 + 8 * D * 2 + SV>(fh[slot], vadr[db]);
    }
  };
  // The fragment stream never drains: after the last K fragment of a tile come the V^T fragments of
  // the next second product, after those the K fragments of the next score tile.  LDS read
  // instructions issued after those of a fragment and before its wait = those of the PD - 1 fragments
  // behind it in that cyclic order (one per K fragment, two per V^T fragment).
  // One wait serves two fragments: the matrix instruction of an even fragment waits until its own
  // reads and those of the odd fragment behind it have landed, the odd one's does not wait (a wait
  // is an instruction of its own in the wavefront's issue stream; the prefetch depth beyond two
  // buys nothing).  An even and the following odd fragment are always of the same kind.
  static_assert(NKF % 2 == 0 && NVF % 2 == 0 && PD >= 3, "");
  auto younger = [](int f) constexpr {
    if (f % 2 != 0) return -1;
    int n = 0;
    for (int r = f + 2; r < f + PD; ++r) n += (r % NF) < NKF ? 1 : 2;
    return n < 15 ? n : 15;
  };
  // ---- vector work dealt out to the matrix instructions of a body.  A matrix instruction keeps
  // its pipe busy for 32 cycles; what the wave issues behind it in that time is free, what exceeds
  // it delays the next one.  The 64 exponentials of a lane (16 per 16-key group, the groups in the
  // order the second product uses them) are spread as evenly as the order allows: PRE before the
  // first matrix instruction (its operand is still on its way from LDS), up to EK under the scores,
  // the rest under the first VE instructions of the second product; the 32 maxima of the next score
  // tile from its instruction VS on.  The instruction after which a tile-fetch load is issued gets
  // no vector work: that load can stall the wave for about as long.
  constexpr int FRAGS_PER_PIECE = NF / (2 * C::PASSES);
  static_assert(NF % (2 * C::PASSES) == 0, "fetch pieces are spread evenly over the fragments");
  constexpr int NE = 32 * NS;                           // exponentials per lane and tile
  constexpr int PRE = 2 * NS, EK = 5 * NE / 8, VE = 3 * NVM / 4, VS = NVM / 4;
  auto is_fetch_slot = [](int m) constexpr { return m % (NS * FRAGS_PER_PIECE) == NS * FRAGS_PER_PIECE - 1; };
  auto work_slots = [is_fetch_slot](int m0, int m1) constexpr { int n = 0; for (int m = m0; m < m1; ++m) n += is_fetch_slot(m) ? 0 : 1; return n; };
  auto vector_slot = [&](auto mm, f32x16 (&S_cur)[NS][2], f32x16 (&S_next)[NS][2]) __attribute__((always_inline)) {
    constexpr int M = decltype(mm)::value;
    if constexpr (!is_fetch_slot(M)) {
      if constexpr (M < NKM) {
        constexpr int n = work_slots(0, NKM), w = work_slots(0, M);
        constexpr int lo = PRE + (EK - PRE) * w / n, hi = PRE + (EK - PRE) * (w + 1) / n;
        static_for<hi - lo>([&](auto i) __attribute__((always_inline)) { exp_one(std::integral_constant<int, lo + decltype(i)::value>{}, S_cur); });
      } else {
        if constexpr (M - NKM < VE) {
          constexpr int n = work_slots(NKM, NKM + VE), w = work_slots(NKM, M);
          constexpr int lo = EK + (NE - EK) * w / n, hi = EK + (NE - EK) * (w + 1) / n;
          static_for<hi - lo>([&](auto i) __attribute__((always_inline)) { exp_one(std::integral_constant<int, lo + decltype(i)::value>{}, S_cur); });
        }
        if constexpr (M - NKM >= VS) {
          constexpr int n = work_slots(NKM + VS, NKM + NVM), w = work_slots(NKM + VS, M);
          constexpr int lo = 16 * NS * w / n, hi = 16 * NS * (w + 1) / n;
          static_for<hi - lo>([&](auto i) __attribute__((always_inline)) { max_step(std::integral_constant<int, lo + decltype(i)::value>{}, S_next); });
        }
      }
    }
  };

  // ---- main loop over 64-key tiles.
  //
  // Body t, entered with the scores S(t+1) (complete but not yet masked), the first part of P(t)
  // and the first V^T fragments of tile t on their way from LDS:
  //   matrix stream:  O^T += V(t)^T P(t)^T                       then   S(t+2) = K(t+2) Q^T
  //   vector stream:  rest of P(t), mask and row maxima of S(t+1);      running max, first part of P(t+1)
  // and it ends at the one barrier of the tile.  Two score tiles alternate, so the loop is unrolled
  // twice; bodies past the last tile work on scores that are all masked (exponentials 0, maxima
  // -inf).  The loop boundary sits in the middle of the dependency chain on purpose: the barrier
  // then falls where the fragments of the next matrix instructions are already in registers or on
  // their way (they belong to tiles that were complete a barrier ago), so the matrix stream runs
  // across it, instead of restarting from an empty pipeline after every barrier.
  //
  // Tile ring (four stages, K half and V half used independently).  K(u) is read in the second half
  // of body u-2, V(u) in the first half of body u (its first fragments at the end of body u-1).
  // Body t, after the barrier that opens it, starts fetch round t+4: K(t+4) - into the stage K(t)
  // left in body t-2 - and V(t+3) - into the stage V(t-1) left in body t-1, which every wavefront
  // has finished, having passed the barrier.  Before a barrier every wavefront waits for its loads
  // of all rounds but the newest, so at the barrier that opens body t the rounds up to t+2 are
  // complete: K up to t+2 and V up to t+1, which is what body t reads.
  //
  // The wavefronts of a SIMD share its issue slots, and when several have an instruction ready the
  // arbiter always takes the one that was launched first: left alone, the first four wavefronts
  // of the workgroup finish a body in 2 700 cycles and wait 700 at the barrier while the other four,
  // which got what slots were left, take 3 300.  So every wavefront lowers its own priority as it
  // moves through a body: whoever is behind outranks whoever is ahead.  At equal priority the
  // older wavefront still wins, so the steps come late and ever closer together (3 up to 5/8 of
  // the body, 2 up to 13/16, 1 up to 15/16, then 0): the stretch before the barrier in which the
  // older one can gain on the younger is short, and they arrive within about sixty cycles of
  // each other (even quarters: two hundred).  No branch is involved.
  constexpr std::integral_constant<int, 1> one_in_flight{};
  // fragment g of the cyclic stream that starts with the V^T fragments of tile tv and goes on with the K fragments of tile tk
  auto issue_cyc = [&](auto gg_, auto sk_, auto sv_) __attribute__((always_inline)) {
    constexpr int G = decltype(gg_)::value;
    if constexpr (G < NVF) issue(std::integral_constant<int, NKF + G>{}, sk_, sv_);
    else issue(std::integral_constant<int, G - NVF>{}, sk_, sv_);
  };
  // the priority ladder of a body (above): position g of its NF matrix instructions
  auto lower_prio = [](auto gg_) __attribute__((always_inline)) {
    constexpr int G = decltype(gg_)::value;
    if constexpr (G == NF * 5 / 8) __builtin_amdgcn_s_setprio(2);
    if constexpr (G == NF * 13 / 16) __builtin_amdgcn_s_setprio(1);
    if constexpr (G == NF * 15 / 16) __builtin_amdgcn_s_setprio(0);
  };
  // Second product of tile t: S_cur = S(t), S_next = S(t+1).  Its trailing reads are the first K fragments of tile t+2.
  // ts_ = t % 4, the ring stage of tile t, at compile time (the loop is unrolled four times).
  auto pv_half = [&](auto ts_, int t, f32x16 (&S_cur)[NS][2], f32x16 (&S_next)[NS][2]) __attribute__((always_inline)) {
    constexpr int TS = decltype(ts_)::value;
    constexpr std::integral_constant<int, (TS + 2) & 3> sk_{};
    constexpr std::integral_constant<int, TS> sv_{};
    static_for<NVF>([&](auto gg_) __attribute__((always_inline)) {
      constexpr int G = decltype(gg_)::value, F = NKF + G, slot = F % PD, W = younger(F);
      constexpr int gg = G / DB, db = G % DB;
      lower_prio(std::integral_constant<int, G>{});
      if constexpr (G == 1) fetch_begin(t + 4, ts_);
      if constexpr (db == 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) fence_p(pf[s][gg]);
      }
      if constexpr (NS * G == VS) {
        // the scores of tile t+1 are complete (several matrix instructions of the second product lie between)
        fence_scores(S_next);
        mask(std::integral_constant<int, (TS + 1) & 3>{}, t + 1, S_next);
      }
      const u32x4 av = {fl[slot][0], fl[slot][1], fh[slot][0], fh[slot][1]};
      static_for<NS>([&](auto ss) __attribute__((always_inline)) {
        constexpr int s = decltype(ss)::value, WW = s == 0 ? W : -1;     // the first strip's instruction waits for the fragment
        mfma_o<ACC, WW>(o[s][db], av, pf[s][gg]);
        vector_slot(std::integral_constant<int, NS * F + s>{}, S_cur, S_next);
        __builtin_amdgcn_sched_barrier(0);
      });
      issue_cyc(std::integral_constant<int, (G + PD) % NF>{}, sk_, sv_);
      if constexpr ((G + 1) % FRAGS_PER_PIECE == 0) fetch_piece((G + 1) / FRAGS_PER_PIECE - 1);
    });
  };
  // Scores of tile t2 into S_next while S_cur = S(t2-1) turns into P(t2-1).  PRIME: nothing is in
  // flight yet (the first call).  Its trailing reads are the first V^T fragments of tile t2-1.
  // (t2s_ = t2 % 4)
  auto qk_half = [&](auto prime, auto t2s_, f32x16 (&S_cur)[NS][2], f32x16 (&S_next)[NS][2]) __attribute__((always_inline)) {
    constexpr bool PRIME = decltype(prime)::value;
    constexpr int T2S = decltype(t2s_)::value;
    constexpr std::integral_constant<int, T2S> sk_{};
    constexpr std::integral_constant<int, (T2S + 3) & 3> sv_{};
    if constexpr (PRIME) static_for<PD>([&](auto f) __attribute__((always_inline)) { issue(f, sk_, sv_); });
    raise_max();                                  // of S_cur
#pragma unroll
    for (int s = 0; s < NS; ++s) {                // what rounding adds to this lane's largest probability of the tile
      const float p_top = fast_exp2(__builtin_fmaf(mx[s], c, -m_run[s]));
      r_fix[s] += static_cast<float>(static_cast<__bf16>(p_top)) - p_top;
    }
    static_for<PRE>([&](auto i) __attribute__((always_inline)) { exp_one(i, S_cur); });
    __builtin_amdgcn_sched_barrier(0);
    static_for<NKF>([&](auto ff) __attribute__((always_inline)) {
      constexpr int F = decltype(ff)::value, slot = F % PD, W = younger(F), G = NVF + F;
      constexpr int ks = F / 2, kb = F % 2;
      if constexpr (!PRIME) lower_prio(std::integral_constant<int, G>{});
      static_for<NS>([&](auto ss) __attribute__((always_inline)) {
        constexpr int s = decltype(ss)::value, WW = s == 0 ? W : -1;
        if constexpr (ks == 0) mfma_s_first<ACC, WW>(S_next[s][kb], fk[slot], qf[s][0]);
        else mfma_s<ACC, WW>(S_next[s][kb], fk[slot], qf[s][ks]);
        vector_slot(std::integral_constant<int, NS * F + s>{}, S_cur, S_next);
        __builtin_amdgcn_sched_barrier(0);
      });
      issue_cyc(std::integral_constant<int, (G + PD) % NF>{}, sk_, sv_);
      if constexpr (!PRIME && (G + 1) % FRAGS_PER_PIECE == 0) fetch_piece((G + 1) / FRAGS_PER_PIECE - 1);
    });
  };
  auto body = [&](auto ts_, int t, f32x16 (&S_a)[NS][2], f32x16 (&S_b)[NS][2]) __attribute__((always_inline)) {
    __builtin_amdgcn_s_setprio(3);
    pv_half(ts_, t, S_a, S_b);
    qk_half(std::false_type{}, std::integral_constant<int, (decltype(ts_)::value + 2) & 3>{}, S_b, S_a);
    wait_fetches(one_in_flight);
    // A bare barrier where it fits: __syncthreads() also drains this wavefront's LDS reads, i.e. the
    // operand fragments just requested for the next tile, and all eight wavefronts would sit out
    // that round trip together.  Nothing needs the drain: a stage is overwritten only after every
    // read of it has fed a matrix instruction that precedes an earlier barrier, and the fragments
    // in flight belong to stages that stay.  (With twelve wavefronts the bare form costs a
    // register the kernel does not have.)
    if constexpr (NW == 12) __syncthreads();
    else __builtin_amdgcn_s_barrier();
  };

  if (n_tiles > 0) {
    fetch_round(0, stage0, false);           // rounds 0 .. 3: K(0 .. 3) and V(0 .. 2)
    fetch_round(1, stage1, true);
    fetch_round(2, stage2, true);
    fetch_round(3, stage3, true);
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  __syncthreads();

  if (n_tiles > 0) {
    f32x16 Sa[NS][2], Sb[NS][2];
    // scores, mask and row maxima of tile 0: no vector work beside them, but the K fragments are
    // read PD ahead as in the loop (one LDS round trip instead of one per fragment)
    static_for<PD>([&](auto f) __attribute__((always_inline)) { issue(f, stage0, stage0); });
    static_for<NKF>([&](auto ff) __attribute__((always_inline)) {
      constexpr int F = decltype(ff)::value, slot = F % PD, ks = F / 2, kb = F % 2;
      constexpr int W = NKF - 1 - F < PD - 1 ? NKF - 1 - F : PD - 1;     // K fragments read after this one
      static_for<NS>([&](auto ss) __attribute__((always_inline)) {
        constexpr int s = decltype(ss)::value, WW = s == 0 ? W : -1;
        if constexpr (ks == 0) mfma_s_first<ACC, WW>(Sa[s][kb], fk[slot], qf[s][0]);
        else mfma_s<ACC, WW>(Sa[s][kb], fk[slot], qf[s][ks]);
      });
      if constexpr (F + PD < NKF) issue(std::integral_constant<int, F + PD>{}, stage0, stage0);
    });
    fence_scores(Sa);
    mask(stage0, 0, Sa);
    static_for<16 * NS>([&](auto i) __attribute__((always_inline)) { max_step(i, Sa); });
    qk_half(std::true_type{}, stage1, Sa, Sb);
    // Unrolled four times: the ring stage of every tile is then a constant of the code, and the
    // stage offsets of all LDS reads sit in their offset fields instead of costing vector additions.
    // An odd pair of bodies follows the loop (a second way out of the loop would do, but then the
    // compiler keeps the wavefront-uniform loop state in vector registers).
    const int n_pairs = (n_tiles + 1) / 2;
    int t = 0;
    for (int q = 0; q < n_pairs / 2; ++q, t += 4) {
      body(stage0, t, Sa, Sb);
      body(stage1, t + 1, Sb, Sa);
      body(stage2, t + 2, Sa, Sb);
      body(stage3, t + 3, Sb, Sa);
      if ((t & 60) == 60) {                      // every 64 tiles
#pragma unroll
        for (int s = 0; s < NS; ++s) { l_run[s] += l_lo[s]; l_lo[s] = 0.f; }
      }
    }
    // The first V^T fragments of the next tile are still on their way into registers.  They are
    // waited for here, where the stream ends; the odd pair of bodies asks for them again (the two
    // paths then join with all registers landed: the compiler may copy them at the join).
    auto drain = [&]() __attribute__((always_inline)) {
      // (inputs only: that keeps the registers reserved up to here and asks for no copies)
      asm volatile("s_waitcnt lgkmcnt(0)" : : "v"(fl[0]), "v"(fl[1]), "v"(fl[2]), "v"(fl[3]), "v"(fh[0]), "v"(fh[1]), "v"(fh[2]), "v"(fh[3]));
    };
    drain();
    if (n_pairs & 1) {
      static_for<PD>([&](auto f) __attribute__((always_inline)) { issue(std::integral_constant<int, NKF + decltype(f)::value>{}, stage2, stage0); });
      body(stage0, t, Sa, Sb);
      body(stage1, t + 1, Sb, Sa);
      drain();
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // no fetch may still be writing LDS when the workgroup ends
  if constexpr (PERSIST) __syncthreads();   //   or when any wavefront starts staging the next item there
  fence_o();

  // ---- epilogue: normalise and store.  A lane owns one query row per strip; per (db, i4) it holds
  // 4 consecutive output columns, and its partner lane (+32) the next 4, so a wavefront writes
  // 32-byte pieces of 32 rows per store and the 16 stores of a lane complete its 512-byte row.
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const float l_mine = l_run[s] + l_lo[s];
    const float l_tot = l_mine + __shfl_xor(l_mine, 32), r_tot = l_tot + (r_fix[s] + __shfl_xor(r_fix[s], 32));
    const bool seen = l_tot > 0.f;
    const float inv = seen && r_tot > 0.f ? 1.f / r_tot : 0.f;
    float lse_new = seen ? (m_run[s] + __builtin_amdgcn_logf(l_tot)) * kLn2 : -__builtin_inff();
    if (q_valid[s]) {
      const int64_t grow = T.q_row0 + my_q[s];
      float* od = p.o_dst + bi * p.o_bstride + (grow * p.Hq + hq) * D + 4 * h;
      float* ld = p.lse_dst + bi * p.lse_bstride + grow * p.Hq + hq;
      float wa = 0.f, wb = inv;
      if (p.merge) {
        // update_out_lse of Algorithm 3 folded into the store
        const float lse_old = *ld;
        const float mxl = fmaxf(lse_old, lse_new);
        if (mxl == -__builtin_inff()) {
          wb = 0.f;
        } else {
          const float ea = __expf(lse_old - mxl), eb = __expf(lse_new - mxl);
          const float rden = 1.f / (ea + eb);
          wa = ea * rden;
          wb = eb * rden * inv;
          lse_new = mxl + __logf(ea + eb);
        }
      }
      // All pieces of the old row are requested before the first one is written back: loads and
      // stores through the same pointer are otherwise kept in program order, one round trip each.
      f32x4 old[DB][4];
      if (p.merge) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) old[db][i4] = *reinterpret_cast<const f32x4*>(od + 32 * db + 8 * i4);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          f32x4 val;
#pragma unroll
          for (int e = 0; e < 4; ++e) val[e] = o[s][db][4 * i4 + e] * wb;
          if (p.merge) {
#pragma unroll
            for (int e = 0; e < 4; ++e) val[e] = __builtin_fmaf(wa, old[db][i4][e], val[e]);
          }
          *reinterpret_cast<f32x4*>(od + 32 * db + 8 * i4) = val;
        }
      if (h == 0) *ld = lse_new;
    }
  }
  }  // next work item (PERSIST)
}

template <int D, int NS, int NW>
hipError_t launch_variant(const AttnLaunch& p0, hipStream_t stream) {
  using C = Cfg<D, NS, NW>;
  int64_t tiles = 0;
  for (int t = 0; t < p0.n_tasks; ++t) tiles += (p0.task[t].n_q + C::BM - 1) / C::BM;
  const int64_t items = tiles * p0.Hq * p0.batch;
  if (items == 0) return hipSuccess;
  if (items > INT_MAX) return hipErrorInvalidValue;
  if constexpr (D == 64 && NW == 8) {          // (twelve wavefronts leave no registers for the outer loop)
    if (p0.seg_ext[0] != nullptr) {            // all steps in one launch: persistent workgroups, one per CU
      int dev = 0, cus = 0;
      if (note_hip(hipGetDevice(&dev)) != hipSuccess ||
          note_hip(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess)
        return hipErrorInvalidValue;
      cus -= cus % 8;
      if (cus >= 8 && items > cus) {
        AttnLaunch p = p0;
        p.n_items = static_cast<int32_t>(items);
        return TASP_LAUNCH((attn_bf16_kernel<D, NS, NW, true>), dim3(static_cast<unsigned>(cus)), dim3(C::NTHREADS), stream, p);
      }
    }
  }
  const AttnLaunch& p = p0;
  const int64_t units = static_cast<int64_t>(p0.batch) * p0.Hkv;
  const int64_t blocks = xcd_balanced_blocks(units, items / units);
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  return TASP_LAUNCH((attn_bf16_kernel<D, NS, NW, false>), dim3(static_cast<unsigned>(blocks)), dim3(C::NTHREADS), stream, p);
}

}  // namespace

// One strip per wavefront (eight wavefronts, two per SIMD) is the faster configuration: with two
// strips the single wavefront of a SIMD has to issue every instruction itself and is bound by that.
hipError_t launch_attn_bf16(const AttnLaunch& p, int d, hipStream_t stream) {
  if (d == 128) return launch_variant<128, 1, 8>(p, stream);
  if (d == 64) {
    // At d = 64 the kernel needs 168 registers, so three wavefronts fit a SIMD (twelve per
    // workgroup, 384 query rows): measured 5-40 % faster than eight when the query blocks fill
    // 384-row tiles as well as 256-row tiles; 3 % more padding already eats the gain.  Where eight
    // are launched and all steps are in one launch, they run as persistent workgroups.
    int64_t rows8 = 0, rows12 = 0;
    for (int t = 0; t < p.n_tasks; ++t) {
      rows8 += (p.task[t].n_q + 255) / 256 * 256;
      rows12 += (p.task[t].n_q + 383) / 384 * 384;
    }
    return rows12 * 100 <= rows8 * 101 ? launch_variant<64, 1, 12>(p, stream) : launch_variant<64, 1, 8>(p, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace tasp
