// Blockwise attention of one step of Algorithm 3 on gfx950: bf16 inputs, fp32 scores/softmax/output.
//
// The paper concatenates the N-1 sub-chunks of a step and calls a flash-attention library on the
// copy (Algorithm 3; Sec. 5.4 puts the cost of that copy at 1-5 % of the compute time).  Here the
// kernel walks the *virtual* concatenation instead: a workgroup owns 32 x NWAVES query rows of one head and
// streams 64-key tiles whose rows are gathered from the K/V segments of the step, so sub-chunk
// lengths that are no tile multiple cost nothing and nothing is copied.
//
// Per wave (32 query rows):  S^T = K Q^T  and  O^T = V^T P^T  with v_mfma_f32_32x32x16_bf16.
// Computing the transposed products puts one query in one lane column, so the row max / row sum of
// the online softmax are in-lane reductions over 32 registers plus one exchange between the two
// lane halves, the rescale factor is a per-lane scalar, and the fp32 -> bf16 P tile is already in
// the B-operand layout of the second product.  K tiles are read from LDS with 16-byte reads, V
// tiles with the transposing LDS read (ds_read_b64_tr_b16); both tiles are XOR-swizzled in 16-byte
// units so that neither the fills nor the reads conflict on banks.
#include <hip/hip_runtime.h>

#include <climits>
#include <type_traits>
#include <utility>

#include "internal.hpp"

namespace tasp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

constexpr int BN = 64;           // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleGap = 8.0f;   // the running max is only raised when it grew by more than 2^8
constexpr float kNegBig = -1.0e30f;

template <int D, int NWAVES>
struct Cfg {
  static constexpr int NTHREADS = 64 * NWAVES;
  static constexpr int BM = 32 * NWAVES;              // query rows per workgroup
  static constexpr int UNITS = D / 8;                 // 16-byte units per row
  static constexpr int LOADERS = 64 * (NWAVES / 2);   // threads that fetch tiles: the first half of the waves
  static constexpr int RPP = LOADERS / UNITS < BN ? LOADERS / UNITS : BN;   // rows filled per pass
  static constexpr int PASSES = BN / RPP;
  static constexpr int ROWS_PER_LINE = 16 / UNITS;    // rows per 256-byte bank line (1 or 2)
  static constexpr int TILE_BYTES = BN * D * 2;
  static constexpr int STAGES = 4;
  static constexpr int SMEM = STAGES * 2 * TILE_BYTES;   // ring of (K tile, V tile)
  __device__ static int swz_k(int row, int unit) { return unit ^ ((row / ROWS_PER_LINE) % UNITS); }
  __device__ static int swz_v(int row, int unit) { return unit ^ (4 * ((row / ROWS_PER_LINE) % (UNITS / 4))); }
};

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// One direct global->LDS load of 16 bytes per lane: lane l's bytes land at lds_base + 16 l.  Written
// as inline assembly so that the wait for it is placed by hand (s_waitcnt vmcnt before the barrier
// that publishes the tile) instead of in front of the next LDS read; no other vector memory
// instruction is in flight while these are.  It carries no memory clobber: the stage it fills is
// not read before the next barrier, and barriers and waits are ordered against volatile assembly.
__device__ inline void dma16(const unsigned char* src, unsigned char* lds_base) {
  const unsigned lds_addr = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)lds_base));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr), "v"(src));
}

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// LDS operand reads whose wait is placed by hand.  The compiler puts an LDS read one or two matrix
// instructions ahead of its use, which leaves most of the LDS latency exposed with two wavefronts
// per SIMD; here the reads of PD operand fragments are kept in flight.  A read is volatile assembly
// (issued in program order), and the fragment reaches its matrix instruction only through lds_wait,
// which waits until at most N younger LDS instructions are outstanding (LDS instructions of a
// wavefront complete in order, so extra ones the compiler adds only make a wait stricter).
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
// marks a fragment as defined after the preceding (volatile) wait
__device__ __forceinline__ void after_wait(u32x4& f) { asm volatile("" : "+v"(f)); }
__device__ __forceinline__ void after_wait(u32x2& a, u32x2& b) { asm volatile("" : "+v"(a), "+v"(b)); }

// Order of the matrix instructions of one loop iteration.  ROLE 0 (first half of the waves):
// K Q^T of tile t, then V^T P^T of tile t.  ROLE 1: V^T P^T of tile t, then K Q^T of tile t+1.
template <int D, int ROLE>
struct Seq {
  static constexpr int NK = 2 * (D / 16);      // matrix instructions of K Q^T per tile (one 16-byte LDS read each)
  static constexpr int NV = 4 * (D / 32);      //   and of V^T P^T (two transposing 8-byte reads each)
  static constexpr int NOPS = NK + NV;
  static constexpr bool is_k(int pos) { return ROLE == 0 ? pos < NK : pos >= NV; }
  static constexpr int idx(int pos) { return ROLE == 0 ? (pos < NK ? pos : pos - NK) : (pos < NV ? pos : pos - NV); }
  static constexpr int tile_off(int pos) { return ROLE == 1 && pos >= NV ? 1 : 0; }
  // LDS reads issued between the read of position q and its wait when pd fragments are kept ahead (the counter holds 15)
  static constexpr int younger(int q, int pd) {
    int n = 0;
    for (int r = q + 1; r <= q + pd; ++r) n += is_k(r % NOPS) ? 1 : 2;
    return n < 15 ? n : 15;
  }
};

template <int D, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES, 2) void attn_bf16_kernel(const AttnLaunch p) {
  using C = Cfg<D, NWAVES>;
  constexpr int BM = C::BM;
  constexpr int KS = D / 16;     // contraction steps of K Q^T
  constexpr int DB = D / 32;     // 32-row blocks of O^T

  __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];   // ring of stages, each a K tile then a V tile
  __shared__ __attribute__((aligned(16))) int s_tok[C::STAGES][BN];   // global position of every key row of a tile (INT_MAX: none)
  __shared__ int e_vbeg[2 * kMaxSeg + 1];  // effective segments: start in the virtual concatenation
  __shared__ int e_goff[2 * kMaxSeg];      //   global position minus virtual position
  __shared__ int e_diag[2 * kMaxSeg];      //   straddles the diagonal of this query tile
  __shared__ int e_n;
  __shared__ int m_lo[2 * kMaxSeg + 2];    // runs of tiles that need the element-wise mask (sorted, the
  __shared__ int m_hi[2 * kMaxSeg + 2];    //   last run is open-ended: m_hi = INT_MAX)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int h = lane >> 5;       // lane half
  const int lq = lane & 31;      // query column inside the wave

  // ---- which (KV head, task, query tile, query head) this workgroup owns.  Workgroups are dealt
  // round-robin to the 8 XCDs; the index is remapped so that each XCD gets a contiguous run of work
  // ordered KV-head-major: the workgroups of one XCD then stream the same K/V through its L2.
  const int G = p.Hq / p.Hkv;
  const int tiles0 = (p.task[0].n_q + BM - 1) / BM;
  const int tiles1 = p.n_tasks > 1 ? (p.task[1].n_q + BM - 1) / BM : 0;
  const int per_g = (tiles0 + tiles1) * G;
  const int nblocks = gridDim.x;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int q8 = nblocks >> 3, r8 = nblocks & 7;
  const int w = xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
  const int g = w / per_g;
  int rem = w - g * per_g;
  const int tsk = rem >= tiles0 * G ? 1 : 0;
  if (tsk) rem -= tiles0 * G;
  const int tile_q = rem / G;
  const int hq = g * G + rem % G;
  const AttnTask& T = p.task[tsk];
  const int q_tile_row0 = tile_q * BM;                        // relative to the task
  const int q_rows_here = min(BM, T.n_q - q_tile_row0);
  const int qa = T.q_pos0 + q_tile_row0;                      // first and last position of the tile
  const int qb = qa + q_rows_here - 1;

  // ---- effective segment list of this query tile: drop what the causal mask hides from every
  // row, split the rest into a part every row sees and a part that straddles the diagonal.
  if (tid == 0) {
    int n = 0, vpos = 0;
    for (int s = 0; s < T.n_seg; ++s) {
      const int a = T.seg_start[s], b = T.seg_end[s];
      if (!p.causal) {
        e_vbeg[n] = vpos; e_goff[n] = a - vpos; e_diag[n] = 0; vpos += b - a; ++n;
        continue;
      }
      if (a > qb) continue;
      const int b_vis = min(b, qb + 1);
      const int full_end = min(b_vis, qa + 1);
      if (a < full_end) { e_vbeg[n] = vpos; e_goff[n] = a - vpos; e_diag[n] = 0; vpos += full_end - a; ++n; }
      const int ds = max(a, full_end);
      if (ds < b_vis) { e_vbeg[n] = vpos; e_goff[n] = ds - vpos; e_diag[n] = 1; vpos += b_vis - ds; ++n; }
    }
    e_vbeg[n] = vpos;
    e_n = n;
    // tiles that touch a diagonal segment, and everything from the first tile that runs past the last key
    int mn = 0;
    for (int j = 0; j < n; ++j) {
      if (!e_diag[j]) continue;
      const int lo = e_vbeg[j] / BN, hi = (e_vbeg[j + 1] - 1) / BN;
      if (mn > 0 && lo <= m_hi[mn - 1]) m_hi[mn - 1] = max(m_hi[mn - 1], hi);
      else { m_lo[mn] = lo; m_hi[mn] = hi; ++mn; }
    }
    const int tail = vpos / BN;
    if (mn > 0 && tail <= m_hi[mn - 1]) m_hi[mn - 1] = INT_MAX;
    else { m_lo[mn] = tail; m_hi[mn] = INT_MAX; ++mn; }
  }
  __syncthreads();
  const int n_eff = e_n;
  const int total_keys = e_vbeg[n_eff];
  const int n_tiles = (total_keys + BN - 1) / BN;

  // ---- Q fragments (B operand of K Q^T): lane holds query lq, d = 16 ks + 8 h .. +8
  const int my_q = q_tile_row0 + wave * 32 + lq;              // row inside the task
  const bool q_valid = my_q < T.n_q;
  const int64_t q_row = T.q_row0 + (q_valid ? my_q : T.n_q - 1);
  bf16x8 qf[KS];
  {
    const __bf16* src = static_cast<const __bf16*>(p.q) + (q_row * p.Hq + hq) * D + 8 * h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(src + 16 * ks);
  }
  // Land the Q fragments now (vmcnt(0)); otherwise their pending loads make the compiler wait on
  // the K/V prefetch of each iteration in front of the first products that read qf.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  const int q_pos = p.causal ? T.q_pos0 + my_q : INT_MAX - 1;

  // ---- loader: this thread fills rows fr + RPP*i, unit fu of every K and V tile.  Byte offsets
  // into K and V fit 32 bits (checked on the host).
  const int fr = tid / C::UNITS, fu = tid % C::UNITS;
  const unsigned row_bytes = static_cast<unsigned>(p.Hkv) * D * 2;
  // Row bookkeeping of the loader.  Each thread follows its PASSES rows through the virtual
  // concatenation: from one tile to the next a row moves 64 keys on and normally stays inside its
  // effective segment (token += 64); only when it runs off the end of the segment is the segment
  // list searched again.  tokk = global position (INT_MAX: past the last key), flagk = the row
  // needs the element-wise mask, lefti = keys from the row to the end of its segment.
  int tokk[C::PASSES], flagk[C::PASSES], segi[C::PASSES], lefti[C::PASSES];
  auto relocate = [&](int i, int v) __attribute__((always_inline)) {
    int j = segi[i];
    while (j < n_eff && v >= e_vbeg[j + 1]) ++j;              // rows only move forward
    segi[i] = j;
    if (j < n_eff) { tokk[i] = v + e_goff[j]; flagk[i] = e_diag[j]; lefti[i] = e_vbeg[j + 1] - v; }
    else { tokk[i] = INT_MAX; flagk[i] = 1; lefti[i] = 1 << 30; }
  };
  // rows of tile t; must be called for t = 0, 1, 2, ... in this order
  auto locate = [&](int t) __attribute__((always_inline)) {
    if (t == 0) {
#pragma unroll
      for (int i = 0; i < C::PASSES; ++i) { segi[i] = 0; relocate(i, fr + C::RPP * i); }
      return;
    }
    bool off_end = false;
#pragma unroll
    for (int i = 0; i < C::PASSES; ++i) {
      lefti[i] -= BN;
      tokk[i] = tokk[i] == INT_MAX ? INT_MAX : tokk[i] + BN;
      off_end |= lefti[i] <= 0;
    }
    if (__builtin_amdgcn_ballot_w64(off_end) != 0) {
#pragma unroll
      for (int i = 0; i < C::PASSES; ++i)
        if (lefti[i] <= 0) relocate(i, t * BN + fr + C::RPP * i);
    }
  };
  // Fetch tile t straight into ring stage `stage` (global_load_lds: no registers, no LDS write
  // instructions).  A wavefront's 64 lanes fill 1 KiB of consecutive LDS; the XOR swizzle of the
  // tile layout is applied on the source side: the lane that owns LDS slot (row, unit) reads the
  // 16 bytes of column swz(row, unit) of that row.  Rows past the end fetch token 0 and are masked.
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned char* Kd = static_cast<const unsigned char*>(p.k) + (static_cast<size_t>(g) * D + C::swz_k(fr, fu) * 8) * 2;
  const unsigned char* Vd = static_cast<const unsigned char*>(p.v) + (static_cast<size_t>(g) * D + C::swz_v(fr, fu) * 8) * 2;
  static_assert(C::RPP % 16 == 0, "the swizzle of a thread's rows must not depend on the pass");
  // A tile fetch is 2*PASSES loads per thread.  The path from L2 into LDS takes roughly 25 cycles per
  // wavefront-load and the issuing wave stalls once its queue is full, so the loads are not issued
  // in one burst: fetch_begin does the bookkeeping, fetch_piece(j) issues load j, and the scores
  // phase drops one piece between its matrix instructions.
  unsigned fetch_off[C::PASSES];
  unsigned char* fetch_dst = smem;
  auto fetch_begin = [&](int t, int stage) __attribute__((always_inline)) {
    locate(t);
    fetch_dst = smem + stage * 2 * C::TILE_BYTES + wave_u * 1024;
#pragma unroll
    for (int i = 0; i < C::PASSES; ++i) {
      fetch_off[i] = __umul24(tokk[i] == INT_MAX ? 0u : static_cast<unsigned>(tokk[i]), row_bytes);   // both below 2^24 (host check)
      if (fu == 0) s_tok[stage][fr + C::RPP * i] = tokk[i];
    }
  };
  auto fetch_piece = [&](int j) __attribute__((always_inline)) {
    const int i = j >> 1;
    if (j & 1) dma16(Vd + fetch_off[i], fetch_dst + C::TILE_BYTES + i * C::LOADERS * 16);
    else dma16(Kd + fetch_off[i], fetch_dst + i * C::LOADERS * 16);
  };
  auto fetch = [&](int t, int stage) __attribute__((always_inline)) {
    fetch_begin(t, stage);
#pragma unroll
    for (int j = 0; j < 2 * C::PASSES; ++j) fetch_piece(j);
  };
  // wait until at most `newest` of this wave's tile fetches (each 2*PASSES loads) are still in flight
  auto wait_fetches = [&](auto newest) __attribute__((always_inline)) {
    constexpr int N = decltype(newest)::value * 2 * C::PASSES;
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  };

  // ---- per-lane LDS read offsets (loop invariant)
  int koff[KS];       // K: row lq (+32 kb), unit 2 ks + h
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = (lq * C::UNITS + C::swz_k(lq, 2 * ks + h)) * 16;
  const unsigned smem_lds = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)smem));
  unsigned kadr[KS];  // the same as LDS addresses, stage 0
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kadr[ks] = smem_lds + koff[ks];
  // V^T through the transposing read: 16-lane group a = lane/16 serves d columns 16 (a%2) .. +16 of
  // a 32-wide block for lane half h = a/2; lane jj of the group points at key 4 h + jj/4, 4 d values.
  const int ga = lane >> 4, jj = lane & 15;
  const int vrow = 4 * (ga >> 1) + (jj >> 2);                 // key row inside a 16-key block (+8 second read)
  int voff[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    const int unit = 4 * db + 2 * (ga & 1) + ((jj & 3) >> 1);
    voff[db] = (vrow * C::UNITS + C::swz_v(vrow, unit)) * 16 + 8 * (jj & 1);
  }
  unsigned vadr[DB];  // LDS addresses inside the V tile of stage 0
#pragma unroll
  for (int db = 0; db < DB; ++db) vadr[db] = smem_lds + C::TILE_BYTES + voff[db];

  // S^T = K Q^T of one K tile, reads left to the compiler (used once, before the loop)
  auto scores = [&](int stage, f32x16 (&s)[2], auto) __attribute__((always_inline)) {
    const unsigned char* kbase = smem + stage * 2 * C::TILE_BYTES;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kbase + kb * 32 * D * 2 + koff[ks]);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
      }
  };

  // ---- running state
  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  float m_run = kNegBig;        // running max in the exp2 domain (scaled scores times log2 e)
  float l_run = 0.f;            // this lane's share of the running sum
  const float c = p.scale * kLog2e;

  // ---- the three phases of a tile, for one wave
  // element-wise mask, only for tiles that touch the diagonal or run past the last key
  int m_idx = 0;
  int m_cur_lo = __builtin_amdgcn_readfirstlane(m_lo[0]), m_cur_hi = __builtin_amdgcn_readfirstlane(m_hi[0]);
  auto mask = [&](int t, f32x16 (&s)[2]) __attribute__((always_inline)) {
    while (t > m_cur_hi) {     // t only grows; the last run never ends
      ++m_idx;
      m_cur_lo = __builtin_amdgcn_readfirstlane(m_lo[m_idx]);
      m_cur_hi = __builtin_amdgcn_readfirstlane(m_hi[m_idx]);
    }
    if (t >= m_cur_lo) {
      const int stage = t & 3;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const i32x4 tk = *reinterpret_cast<const i32x4*>(&s_tok[stage][32 * kb + 8 * i4 + 4 * h]);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (tk[e] > q_pos) s[kb][4 * i4 + e] = -__builtin_inff();
        }
    }
  };
  // online softmax (exp2 domain): raises the running max lazily, returns P as bf16 B-operand fragments
  auto softmax = [&](f32x16 (&s)[2], bf16x8 (&pf)[2][2]) __attribute__((always_inline)) {
    float mx = s[0][0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[0][i]);
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[1][i]);
    {
      // the other half of the keys sits in the lane 32 away
      const unsigned mu = __builtin_bit_cast(unsigned, mx);
      const u32x2 sw = __builtin_amdgcn_permlane32_swap(mu, mu, false, false);
      mx = fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1]));
    }
    const float m_cand = fmaxf(m_run, mx * c);
    if (__builtin_amdgcn_ballot_w64(m_cand > m_run + kRescaleGap) != 0) {
      const float alpha = fast_exp2(m_run - m_cand);
      m_run = m_cand;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
    float lsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pv = fast_exp2(__builtin_fmaf(s[kb][i], c, -m_run));
        lsum += pv;
        pf[kb][i >> 3][i & 7] = static_cast<__bf16>(pv);
      }
    l_run += lsum;
  };
  // ---- the matrix instructions of an iteration as one stream of operand fragments: the LDS reads
  // of the fragment PD positions ahead are issued right after the matrix instruction of a position, so
  // the reads run through the phase changes (the first fragments of the second product land while
  // the softmax runs) and into the first products of the next iteration.
  constexpr int PD = 8;
  using SeqA = Seq<D, 0>;
  constexpr int NK = SeqA::NK, NV = SeqA::NV, NOPS = SeqA::NOPS;
  static_assert(NOPS % PD == 0 && NK >= PD && NV >= PD, "fragment ring must close over an iteration");
  u32x4 fk[PD];            // K fragments in flight (ring slot = position % PD)
  u32x2 fl[PD], fh[PD];    // V^T fragments in flight, low and high half
  // issue the reads of stream position Q (may lie in the next iteration); base_* = ring stage byte offsets of tiles t, t+1
  auto issue = [&](auto role, auto qq, unsigned base_cur, unsigned base_next) __attribute__((always_inline)) {
    using S = Seq<D, decltype(role)::value>;
    constexpr int Q = decltype(qq)::value;
    constexpr int pos = Q % NOPS, adv = Q / NOPS + S::tile_off(pos), slot = Q % PD, i = S::idx(pos);
    static_assert(adv <= 1, "only tiles t and t+1 are read");
    const unsigned base = adv ? base_next : base_cur;
    if constexpr (S::is_k(pos)) {
      constexpr int ks = i / 2, kb = i % 2;
      lds_read_b128<kb * 32 * D * 2>(fk[slot], kadr[ks] + base);
    } else {
      constexpr int g = i / DB, db = i % DB;    // 16-key group, 32-row block of O^T
      lds_read_tr_b64<g * 16 * D * 2>(fl[slot], vadr[db] + base);
      lds_read_tr_b64<g * 16 * D * 2 + 8 * D * 2>(fh[slot], vadr[db] + base);
    }
  };
  // wait for the fragment of position Q and run its matrix instruction
  auto exec = [&](auto role, auto qq, f32x16 (&s)[2], const bf16x8 (&pf)[2][2]) __attribute__((always_inline)) {
    using S = Seq<D, decltype(role)::value>;
    constexpr int Q = decltype(qq)::value;
    constexpr int slot = Q % PD, i = S::idx(Q), W = S::younger(Q, PD - 1);
    if constexpr (S::is_k(Q)) {
      constexpr int ks = i / 2, kb = i % 2;
      lds_wait<W>(fk[slot]);
      const bf16x8 a = __builtin_bit_cast(bf16x8, fk[slot]);
      if constexpr (ks == 0) {
        f32x16 z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.f;
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0], z, 0, 0, 0);
      } else {
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
      }
    } else {
      constexpr int g = i / DB, db = i % DB;
      lds_wait<W>(fl[slot], fh[slot]);
      const u32x4 av = {fl[slot][0], fl[slot][1], fh[slot][0], fh[slot][1]};
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pf[g / 2][g % 2], o[db], 0, 0, 0);
    }
  };
  // Fragments that cross the loop edge are waited for before the closing barrier, where the wave
  // waits anyway: a register copy the compiler may place on the loop edge then copies landed data.
  auto land_k = [&]() __attribute__((always_inline)) {
    lds_wait<0>(fk[0]);
    static_for<PD - 1>([&](auto i) __attribute__((always_inline)) { after_wait(fk[decltype(i)::value + 1]); });
  };
  auto land_v = [&]() __attribute__((always_inline)) {
    lds_wait<0>(fl[0], fh[0]);
    static_for<PD - 1>([&](auto i) __attribute__((always_inline)) { after_wait(fl[decltype(i)::value + 1], fh[decltype(i)::value + 1]); });
  };
  constexpr unsigned STAGE_BYTES = 2 * C::TILE_BYTES;

  // ---- main loop over 64-key tiles.  Ring of four LDS stages filled by direct global->LDS loads:
  // at the barrier that opens iteration t, tiles t and t+1 are complete, tile t+2 is in flight and
  // the first half of the waves starts the fetch of tile t+3 into the stage tile t-1 has left;
  // before the barrier that closes the iteration they wait for tile t+2.
  //
  // The two wavefronts that share a SIMD run half an iteration apart: the first goes
  // scores(t) -> softmax -> accumulate(t), the second softmax -> accumulate(t) -> scores(t+1), so
  // that one of them has matrix work while the other is in its vector phase.
  constexpr std::integral_constant<int, 1> one_in_flight{};
  constexpr std::integral_constant<int, 0> role_a{};
  constexpr std::integral_constant<int, 1> role_b{};
  constexpr int OPS_PER_PIECE = NOPS / (2 * C::PASSES);
  static_assert(NOPS % (2 * C::PASSES) == 0, "fetch pieces are spread evenly over the matrix instructions");
  if (n_tiles > 0 && __builtin_amdgcn_readfirstlane(wave) < NWAVES / 2) {
    fetch(0, 0);
    fetch(1, 1);
    fetch(2, 2);
    wait_fetches(one_in_flight);
  }
  __syncthreads();

  if (n_tiles > 0) {
    if (__builtin_amdgcn_readfirstlane(wave) < NWAVES / 2) {
      static_for<PD>([&](auto q) __attribute__((always_inline)) { issue(role_a, q, 0u, STAGE_BYTES); });
      land_k();
      for (int t = 0; t < n_tiles; ++t) {
        fetch_begin(t + 3, (t + 3) & 3);
        f32x16 s[2];
        bf16x8 pf[2][2];
        const unsigned base_cur = (t & 3) * STAGE_BYTES, base_next = ((t + 1) & 3) * STAGE_BYTES;
        static_for<NOPS>([&](auto q) __attribute__((always_inline)) {
          constexpr int Q = decltype(q)::value;
          exec(role_a, q, s, pf);
          issue(role_a, std::integral_constant<int, Q + PD>{}, base_cur, base_next);   // into the ring slot just consumed
          if constexpr ((Q + 1) % OPS_PER_PIECE == 0) fetch_piece((Q + 1) / OPS_PER_PIECE - 1);
          if constexpr (Q == NK - 1) {
            mask(t, s);
            softmax(s, pf);
          }
        });
        wait_fetches(one_in_flight);
        land_k();
        __syncthreads();
      }
    } else {
      f32x16 s[2];
      scores(0, s, std::false_type{});
      static_for<PD>([&](auto q) __attribute__((always_inline)) { issue(role_b, q, 0u, STAGE_BYTES); });
      land_v();
      for (int t = 0; t < n_tiles; ++t) {
        bf16x8 pf[2][2];
        mask(t, s);
        softmax(s, pf);
        const unsigned base_cur = (t & 3) * STAGE_BYTES, base_next = ((t + 1) & 3) * STAGE_BYTES;
        static_for<NOPS>([&](auto q) __attribute__((always_inline)) {
          constexpr int Q = decltype(q)::value;
          exec(role_b, q, s, pf);     // tile t+1 for the scores; past the last tile that is a fetched dummy tile and is dropped
          issue(role_b, std::integral_constant<int, Q + PD>{}, base_cur, base_next);
        });
        land_v();
        __syncthreads();
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // no fetch may still be writing LDS when the workgroup ends

  // ---- epilogue: normalise and store.  A lane owns one query row; per (db, i4) it holds 4
  // consecutive output columns, and its partner lane (+32) the next 4, so a wavefront writes
  // 32-byte pieces of 32 rows per store and the 16 stores of a lane complete its 512-byte row.
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const bool seen = l_tot > 0.f;
  const float inv = seen ? 1.f / l_tot : 0.f;
  float lse_new = seen ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -__builtin_inff();
  if (q_valid) {
    const int64_t grow = T.q_row0 + my_q;
    float* od = p.o_dst + (grow * p.Hq + hq) * D + 4 * h;
    float* ld = p.lse_dst + grow * p.Hq + hq;
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
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        f32x4* dst = reinterpret_cast<f32x4*>(od + 32 * db + 8 * i4);
        f32x4 val;
#pragma unroll
        for (int e = 0; e < 4; ++e) val[e] = o[db][4 * i4 + e] * wb;
        if (p.merge) {
          const f32x4 old = *dst;
#pragma unroll
          for (int e = 0; e < 4; ++e) val[e] = __builtin_fmaf(wa, old[e], val[e]);
        }
        *dst = val;
      }
    if (h == 0) *ld = lse_new;
  }
}

template <int D, int NWAVES>
hipError_t launch_variant(const AttnLaunch& p, hipStream_t stream) {
  constexpr int BM = Cfg<D, NWAVES>::BM;
  int64_t tiles = 0;
  for (int t = 0; t < p.n_tasks; ++t) tiles += (p.task[t].n_q + BM - 1) / BM;
  const int64_t blocks = tiles * p.Hq;
  if (blocks == 0) return hipSuccess;
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  return TASP_LAUNCH((attn_bf16_kernel<D, NWAVES>), dim3(static_cast<unsigned>(blocks)), dim3(64 * NWAVES), stream, p);
}

}  // namespace

hipError_t launch_attn_bf16(const AttnLaunch& p, int d, hipStream_t stream) {
  if (d == 128) return launch_variant<128, 8>(p, stream);
  if (d == 64) return launch_variant<64, 8>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace tasp
