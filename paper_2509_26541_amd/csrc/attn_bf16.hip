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

template <int D, int NWAVES>
__global__ __launch_bounds__(64 * NWAVES, 2) void attn_bf16_kernel(const AttnLaunch p) {
  using C = Cfg<D, NWAVES>;
  constexpr int BM = C::BM;
  constexpr int KS = D / 16;     // contraction steps of K Q^T
  constexpr int DB = D / 32;     // 32-row blocks of O^T

  __shared__ __attribute__((aligned(16))) unsigned char smem[C::SMEM];   // ring of stages, each a K tile then a V tile
  __shared__ __attribute__((aligned(16))) int s_tok[C::STAGES][BN];   // global position of every key row of a tile (INT_MAX: none)
  __shared__ int s_flag[C::STAGES][BN];          // 1: the row needs the element-wise mask
  __shared__ int e_vbeg[2 * kMaxSeg + 1];  // effective segments: start in the virtual concatenation
  __shared__ int e_goff[2 * kMaxSeg];      //   global position minus virtual position
  __shared__ int e_diag[2 * kMaxSeg];      //   straddles the diagonal of this query tile
  __shared__ int e_n;

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
      if (fu == 0) { s_tok[stage][fr + C::RPP * i] = tokk[i]; s_flag[stage][fr + C::RPP * i] = flagk[i]; }
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

  // S^T = K Q^T for the K tile in `kslot`: two 32-key blocks, the two accumulation chains interleaved
  auto scores = [&](int stage, f32x16 (&s)[2], auto with_fetch) __attribute__((always_inline)) {
    const unsigned char* kbase = smem + stage * 2 * C::TILE_BYTES;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kbase + kb * 32 * D * 2 + koff[ks]);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
      }
      if constexpr (decltype(with_fetch)::value) {
        // the first half of the 2*PASSES pieces, spread over the KS steps
#pragma unroll
        for (int j = ks * C::PASSES / KS; j < (ks + 1) * C::PASSES / KS; ++j) fetch_piece(j);
      }
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
  auto mask = [&](int stage, f32x16 (&s)[2]) __attribute__((always_inline)) {
    if (__builtin_amdgcn_ballot_w64(s_flag[stage][lane] != 0) != 0) {
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
    mx = fmaxf(mx, __shfl_xor(mx, 32));
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
  // O^T += V^T P^T : per 16-key block, DB blocks of 32 output rows
  auto accumulate = [&](int stage, const bf16x8 (&pf)[2][2], auto with_fetch) __attribute__((always_inline)) {
    const unsigned char* vbase = smem + (stage * 2 + 1) * C::TILE_BYTES;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const unsigned char* vb = vbase + (32 * kb + 16 * j) * D * 2;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(vb + voff[db]));
          const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(vb + 8 * D * 2 + voff[db]));
          const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kb][j], o[db], 0, 0, 0);
        }
        if constexpr (decltype(with_fetch)::value) {
          // the second half of the pieces, spread over the four 16-key groups
          constexpr int G4 = 4;
          const int grp = 2 * kb + j;
#pragma unroll
          for (int q = C::PASSES + grp * C::PASSES / G4; q < C::PASSES + (grp + 1) * C::PASSES / G4; ++q) fetch_piece(q);
        }
      }
  };

  // ---- main loop over 64-key tiles.  Ring of four LDS stages filled by direct global->LDS loads:
  // at the barrier that opens iteration t, tiles t and t+1 are complete, tile t+2 is in flight and
  // every wave starts the fetch of tile t+3 into the stage tile t-1 has left; before the barrier
  // that closes the iteration it waits for its own part of tile t+2.
  //
  // The two wavefronts that share a SIMD run the same phases half an iteration apart: the first
  // (waves 0..NWAVES/2-1) goes  fetch -> scores(t) -> softmax -> accumulate(t),  the second
  // softmax -> accumulate(t) -> fetch -> scores(t+1).  After each barrier one of them is in a
  // matrix phase while the other is in its vector or loader phase.
  constexpr std::integral_constant<int, 1> one_in_flight{};
  if (n_tiles > 0 && __builtin_amdgcn_readfirstlane(wave) < NWAVES / 2) {
    fetch(0, 0);
    fetch(1, 1);
    fetch(2, 2);
    wait_fetches(one_in_flight);
  }
  __syncthreads();

  if (__builtin_amdgcn_readfirstlane(wave) < NWAVES / 2) {
    for (int t = 0; t < n_tiles; ++t) {
      const int stage = t & 3;
      fetch_begin(t + 3, (t + 3) & 3);
      f32x16 s[2];
      bf16x8 pf[2][2];
      scores(stage, s, std::true_type{});
      mask(stage, s);
      softmax(s, pf);
      accumulate(stage, pf, std::true_type{});
      wait_fetches(one_in_flight);
      __syncthreads();
    }
  } else {
    f32x16 s[2];
    if (n_tiles > 0) scores(0, s, std::false_type{});
    for (int t = 0; t < n_tiles; ++t) {
      const int stage = t & 3;
      bf16x8 pf[2][2];
      mask(stage, s);
      softmax(s, pf);
      accumulate(stage, pf, std::false_type{});
      scores((t + 1) & 3, s, std::false_type{});    // tile t+1; past the last tile this reads a fetched dummy tile and is dropped
      __syncthreads();
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
