// Backward pass of one step of the chunked attention on gfx950: bf16 inputs, fp32 accumulation.
//
// The paper measures the forward pass (Sec. 5.1.2); the backward pass of a rank is the gradient of
// the same computation and visits the KV sub-chunks in the same arrival order (Algorithm 3).  With
// the final lse of the forward pass the probabilities of any (query, key) pair can be recomputed on
// their own,  p = exp(scale q.k - lse),  so a step needs nothing from the other steps:
//     delta_i = sum_d dout_i out_i                      (once per call)
//     ds_ij   = p_ij (dout_i . v_j - delta_i)
//     dq_i   += scale sum_j ds_ij k_j                   (accumulated over the steps)
//     dk_j    = scale sum_i ds_ij q_i,   dv_j = sum_i p_ij dout_i      (complete after the key's step)
//
// Two kernels per step, both built the same way.  One operand pair is stationary: a wavefront keeps
// the rows of 32 queries (Q, dout) or of 32 keys (K, V) in registers as B operands.  The other pair
// is streamed through LDS in 64-row tiles (direct global->LDS loads, two stages).  With X the
// stationary and Y the streamed side the products are
//     T1 = Y1 X1^T,  T2 = Y2 X2^T      (scores and dout.v, one stationary row per lane column)
//     acc += Y^T E                     (E = ds or p in bf16, already in B-operand layout)
// all with v_mfma_f32_32x32x16_bf16; Y is read from LDS both row-wise (16-byte reads) and
// transposed (ds_read_b64_tr_b16) out of the same tile, whose 16-byte units are XOR-swizzled so
// that neither read pattern conflicts on banks.
//   dq kernel:  X = (Q, dout) of 128 queries per workgroup, Y = (K, V) tiles of the step's keys the
//               query tile can see, E = ds^T, acc = dq^T.
//   dkv kernel: X = (K, V) of 128 keys of the step per workgroup, Y = (Q, dout) tiles of every query
//               head of the group and every local query row that can see them, E = p and ds,
//               acc = dv^T and dk^T.
// Sub-chunk lengths are no tile multiples, so both walk a virtual concatenation of key ranges and
// gather rows, as the forward kernel does.
#include <hip/hip_runtime.h>

#include <climits>

#include "gfx950.hpp"
#include "internal.hpp"

namespace tasp {
namespace {

constexpr int BT = 64;             // streamed rows per tile
constexpr float kLog2e = 1.4426950408889634f;

template <int D, int NW>
struct BCfg {
  static constexpr int NTHREADS = 64 * NW;
  static constexpr int BS = 32 * NW;                    // stationary rows per workgroup (32 per wavefront)
  static constexpr int UNITS = D / 8;                   // 16-byte units per row
  static constexpr int RPP = NTHREADS / UNITS;          // rows filled per pass
  static constexpr int PASSES = BT / RPP;
  static constexpr int ROWS_PER_LINE = 16 / UNITS;      // rows per 256-byte bank line (1 or 2)
  static constexpr int TILE_BYTES = BT * D * 2;
  static constexpr int STAGE_BYTES = 2 * TILE_BYTES;    // (Y1 tile, Y2 tile)
  // Physical unit of logical unit `unit` of row `row`.  x counts bank lines; the XOR value is a
  // bijection of 16 consecutive lines (row-wise reads: 32 lanes, one row each, same logical unit)
  // and differs in its upper bits between neighbouring lines (transposed reads: 4 rows, 2 units).
  __device__ static int swz(int row, int unit) {
    const int x = (row / ROWS_PER_LINE) % UNITS;
    return unit ^ ((x % (UNITS / 4)) * 4 + x / (UNITS / 4));
  }
};

// Tile fetches: direct global->LDS loads with a compiler-level fence (the LDS reads here are
// ordinary loads); every use is followed by s_waitcnt vmcnt(0) and a barrier before the tile is read.
__device__ inline void dma16(const unsigned char* base, unsigned off, unsigned char* lds_base) {
  global_to_lds_16<true>(base, off, lds_base);
}
__device__ inline void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ inline bf16x8 lds_row8(const unsigned char* p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(p));
}
// A operand of Y^T E: 32 columns of Y (rows of Y^T) by 16 rows of Y, from two transposing reads
// eight rows apart.
__device__ inline bf16x8 lds_tr8(const unsigned char* lo, const unsigned char* hi) {
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_void_ptr)const_cast<unsigned char*>(lo));
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_void_ptr)const_cast<unsigned char*>(hi));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}
__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ inline unsigned pack2(float lo, float hi) {
  const bf16x2 pk = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
  return __builtin_bit_cast(unsigned, pk);
}

// Per-lane byte offsets inside a tile for the two LDS read patterns.
template <int D>
struct ReadAddr {
  using C = BCfg<D, 4>;      // the swizzle does not depend on the number of wavefronts
  unsigned row[D / 16];        // row lq (+32 per block), logical unit 2 ks + h
  unsigned tr[D / 32][2];      // transposed: 16-row group at +16 rows per group, rows +0 and +8
  __device__ void init(int lane) {
    const int lq = lane & 31, h = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) row[ks] = (lq * C::UNITS + C::swz(lq, 2 * ks + h)) * 16;
    // 16-lane group a = lane/16 serves columns 16 (a%2) .. +16 of a 32-wide block for lane half
    // a/2; lane jj of the group points at row 4 (a/2) + jj/4, 4 columns.
    const int ga = lane >> 4, jj = lane & 15;
    const int r0 = 4 * (ga >> 1) + (jj >> 2);
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      const int unit = 4 * db + 2 * (ga & 1) + ((jj & 3) >> 1);
      tr[db][0] = (r0 * C::UNITS + C::swz(r0, unit)) * 16 + 8 * (jj & 1);
      tr[db][1] = ((r0 + 8) * C::UNITS + C::swz(r0 + 8, unit)) * 16 + 8 * (jj & 1);
    }
  }
};

// ------------------------------------------------------------------------------------------------
// dq kernel
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, D == 64 ? 3 : 2) void bwd_dq_kernel(const BwdLaunch p) {
  using C = BCfg<D, 4>;
  constexpr int KS = D / 16, DB = D / 32, BS = C::BS, NTHREADS = C::NTHREADS;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * C::STAGE_BYTES];   // stage: K tile, V tile
  __shared__ __attribute__((aligned(16))) int s_tok[2][BT];   // global position of every key row (INT_MAX: none)
  __shared__ __attribute__((aligned(16))) int s_msk[2][4];    // per loading wavefront: the tile holds a key some query row of the workgroup must not see
  __shared__ int e_vbeg[kMaxSegAll + 1];   // effective segments: start in the virtual concatenation
  __shared__ int e_goff[kMaxSegAll];       //   global position minus virtual position
  __shared__ int e_n;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, lq = lane & 31;

  // ---- which (sequence, KV head, task, query tile, query head): KV-head-major inside an XCD
  const int G = p.Hq / p.Hkv;
  const int tiles0 = (p.task[0].n_q + BS - 1) / BS;
  const int tiles1 = p.n_tasks > 1 ? (p.task[1].n_q + BS - 1) / BS : 0;
  const int per_g = (tiles0 + tiles1) * G, per_b = per_g * p.Hkv;
  const int w_all = xcd_balanced(blockIdx.x, p.batch * p.Hkv, per_g);
  if (w_all < 0) return;
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
  const int q_tile_row0 = tile_q * BS;
  const int q_rows_here = min(BS, T.n_q - q_tile_row0);
  const int q_last = T.q_pos0 + q_tile_row0 + q_rows_here - 1;
  const int q_first = p.causal ? T.q_pos0 + q_tile_row0 : INT_MAX - 1;   // a key at or before it is seen by every row

  // ---- effective segments of this query tile: drop what the causal mask hides from every row.
  // The list - from the descriptor, or with all steps in one launch from device memory - is
  // staged in the (still unused) tile stages first.  The first wavefront builds the list, 64 segments per round: every
  // lane clips one segment, the positions are running sums (wavefront scans).
  const int32_t* seg_ext = p.seg_ext[tsk];
  int* seg_raw = reinterpret_cast<int*>(smem);
  if (seg_ext != nullptr) {
    for (int i = tid; i < 2 * T.n_seg; i += NTHREADS) seg_raw[i] = seg_ext[i];
  } else if (tid < T.n_seg) {
    seg_raw[2 * tid] = T.seg_start[tid];
    seg_raw[2 * tid + 1] = T.seg_end[tid];
  }
  __syncthreads();
  if (wave == 0) {
    int n_base = 0, v_base = 0;
    for (int s0 = 0; s0 < T.n_seg; s0 += 64) {
      const int s = s0 + lane;
      int a = 0, len = 0;
      if (s < T.n_seg) {
        a = seg_raw[2 * s];
        const int e = seg_raw[2 * s + 1];
        len = max(0, (p.causal ? min(e, q_last + 1) : e) - a);
      }
      const int cnt = len > 0 ? 1 : 0;
      int sc = cnt, sl = len;                      // inclusive scans
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int t1 = __shfl_up(sc, o), t2 = __shfl_up(sl, o);
        if (lane >= o) { sc += t1; sl += t2; }
      }
      if (len > 0) {
        const int idx = n_base + sc - 1, vpos = v_base + sl - len;
        e_vbeg[idx] = vpos; e_goff[idx] = a - vpos;
      }
      n_base += __shfl(sc, 63); v_base += __shfl(sl, 63);
    }
    if (lane == 0) { e_vbeg[n_base] = v_base; e_n = n_base; }
  }
  __syncthreads();
  const int n_eff = e_n;
  const int total_keys = e_vbeg[n_eff];
  const int n_tiles = (total_keys + BT - 1) / BT;

  // ---- stationary side: this lane's query (column lq of the wave's strip), d = 16 ks + 8 h .. +8
  const int my_q = q_tile_row0 + wave * 32 + lq;
  const bool q_valid = my_q < T.n_q;
  const int64_t q_row = T.q_row0 + (q_valid ? my_q : T.n_q - 1);
  const int64_t qoff = bi * p.q_bstride + (q_row * p.Hq + hq) * D;
  bf16x8 qf[KS], dof[KS];
  {
    const __bf16* qs = static_cast<const __bf16*>(p.q) + qoff + 8 * h;
    const __bf16* ds = static_cast<const __bf16*>(p.dout) + qoff + 8 * h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(qs + 16 * ks);
      dof[ks] = *reinterpret_cast<const bf16x8*>(ds + 16 * ks);
    }
  }
  const int64_t loff = bi * p.lse_bstride + q_row * p.Hq + hq;
  // -lse log2(e) and -delta of the row (the arrays hold -lse / scale and -delta).  A row that saw no
  // key (-inf there) or does not exist contributes nothing: exp2(-inf) = 0.
  const float c = p.scale * kLog2e;
  float nl2 = q_valid ? p.nlse[loff] * c : -__builtin_inff();
  float nd = p.ndelta[loff];
  const int q_pos = p.causal ? T.q_pos0 + my_q : INT_MAX - 1;

  // ---- loader: this thread fills rows fr + RPP i, physical unit fu of the K and the V tile
  const int fr = tid / C::UNITS, fu = tid % C::UNITS;
  const unsigned row_bytes = static_cast<unsigned>(p.Hkv) * D * 2;
  const unsigned col = C::swz(fr, fu) * 16;    // the same for every pass: RPP is a multiple of 16
  static_assert(C::RPP % 16 == 0, "");
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned char* Kg = static_cast<const unsigned char*>(p.k) + (bi * p.kv_bstride + static_cast<int64_t>(g) * D) * 2;
  const unsigned char* Vg = static_cast<const unsigned char*>(p.v) + (bi * p.kv_bstride + static_cast<int64_t>(g) * D) * 2;
  // Row bookkeeping as in the forward kernel: a wavefront-load covers RW consecutive rows of the
  // tile, and while these are consecutive keys of one effective segment everything about them is
  // wavefront-uniform (w_tok = global position of the first, w_left = keys from it to the end of its
  // segment, w_seg = the segment): the loads take the row's byte offset as their scalar offset and
  // a lane constant, and nothing is searched.  Otherwise every lane finds its own row.
  constexpr int RW = 64 / C::UNITS;
  const int r_lane = lane / C::UNITS;
  const unsigned lane_const = static_cast<unsigned>(r_lane) * row_bytes + col;
  const u32x4 k_buf = raw_buffer(Kg), v_buf = raw_buffer(Vg);
  int w_tok[C::PASSES], w_left[C::PASSES], w_seg[C::PASSES];
#pragma unroll
  for (int i = 0; i < C::PASSES; ++i) { w_tok[i] = 0; w_left[i] = 0; w_seg[i] = 0; }
  int any_hidden = 0;
  auto fetch_pass = [&](auto ii, int t, int stage) __attribute__((always_inline)) {
    constexpr int i = decltype(ii)::value;
    unsigned char* dst = smem + stage * C::STAGE_BYTES + wave_u * 1024;
    if constexpr (i == 0) any_hidden = 0;
    {
      const int r = fr + C::RPP * i;
      w_left[i] -= BT;                                      // tile 0: from 0, i.e. search
      w_tok[i] += BT;
      asm volatile("" : "+s"(w_tok[i]), "+s"(w_left[i]));   // (kept in scalar registers)
      if (__builtin_expect(w_left[i] >= RW, 1)) {
        s_tok[stage][r] = w_tok[i] + r_lane;                // the UNITS lanes of a row write the same value
        any_hidden |= w_tok[i] + RW - 1 > q_first ? 1 : 0;
        const unsigned soff = static_cast<unsigned>(w_tok[i]) * row_bytes;
        buffer_to_lds_16<true>(k_buf, soff, lane_const, dst + i * NTHREADS * 16);
        buffer_to_lds_16<true>(v_buf, soff, lane_const, dst + C::TILE_BYTES + i * NTHREADS * 16);
      } else {
        const int v = t * BT + r;
        int j = w_seg[i];
        while (j < n_eff && v >= e_vbeg[j + 1]) ++j;       // rows only move forward
        const int tok = j < n_eff ? v + e_goff[j] : INT_MAX;
        const int left = j < n_eff ? e_vbeg[j + 1] - v : 0;   // past the last key: searched again next time
        w_tok[i] = __builtin_amdgcn_readfirstlane(tok);
        w_left[i] = __builtin_amdgcn_readfirstlane(left);
        w_seg[i] = __builtin_amdgcn_readfirstlane(j);
        any_hidden |= __builtin_amdgcn_ballot_w64(tok > q_first) != 0 ? 1 : 0;
        s_tok[stage][r] = tok;
        const unsigned off = (tok == INT_MAX ? 0u : static_cast<unsigned>(tok)) * row_bytes + col;
        buffer_to_lds_16<true>(k_buf, 0u, off, dst + i * NTHREADS * 16);
        buffer_to_lds_16<true>(v_buf, 0u, off, dst + C::TILE_BYTES + i * NTHREADS * 16);
      }
    }
    if constexpr (i == C::PASSES - 1) { if (lane == 0) s_msk[stage][wave] = any_hidden; }
  };
  auto fetch = [&](int t, int stage) __attribute__((always_inline)) {
    static_for<C::PASSES>([&](auto ii) __attribute__((always_inline)) { fetch_pass(ii, t, stage); });
  };

  ReadAddr<D> ra;
  ra.init(lane);

  f32x16 dq[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

  constexpr int NFB = 2 * KS + 2 * DB, NFT = 2 * NFB, PD = 3;
  bf16x8 ring[PD];        // operand fragments in flight (slot = fragment % PD)
  auto issue = [&](auto ff, const unsigned char* kt, const unsigned char* vt) __attribute__((always_inline)) {
    constexpr int F = decltype(ff)::value, kb = F / NFB, f = F % NFB, slot = F % PD;
    if constexpr (f < KS) {
      ring[slot] = lds_row8(kt + ra.row[f] + kb * 32 * D * 2);
    } else if constexpr (f < 2 * KS) {
      ring[slot] = lds_row8(vt + ra.row[f - KS] + kb * 32 * D * 2);
    } else {
      constexpr int j = (f - 2 * KS) / DB, db = (f - 2 * KS) % DB, grp = (2 * kb + j) * 16 * D * 2;
      ring[slot] = lds_tr8(kt + ra.tr[db][0] + grp, kt + ra.tr[db][1] + grp);
    }
  };

  if (n_tiles > 0) fetch(0, 0);
  // The compiler cannot see the hand-written waits on the tile fetches; left alone it waits inside
  // the loop for the loads of the stationary rows again, before the instructions that read them,
  // and in hardware those waits hit the fetch of the next tile.  Using the values here ends that.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]), "+v"(dof[ks]));
  asm volatile("" : "+v"(nl2), "+v"(nd));
  for (int t = 0; t < n_tiles; ++t) {
    const int stage = t & 1;
    wait_all_loads();
    __syncthreads();                 // tile t is complete; nobody reads the other stage any more
    const bool more = t + 1 < n_tiles;
    const unsigned char* kt = smem + stage * C::STAGE_BYTES;
    const unsigned char* vt = kt + C::TILE_BYTES;
    // most tiles are seen completely by every row: the element-wise mask is skipped for them
    const i32x4 mk = *reinterpret_cast<const i32x4*>(&s_msk[stage][0]);
    const bool need_mask = __builtin_amdgcn_readfirstlane(mk[0] | mk[1] | mk[2] | mk[3]) != 0;
    // The matrix instructions of a tile as one stream of operand fragments, per 32-key block kb:
    // KS row fragments of K (scores), KS of V (dout.v), 2 DB transposed fragments of K (dq).  The
    // read of fragment F + PD is issued right after the instruction that consumed fragment F; the
    // scheduling barrier after every instruction keeps that order (the compiler still places the
    // waits itself: these are ordinary loads).  p is formed under the dout.v instructions, ds for
    // the second 16 keys under the first dq instructions.
    f32x16 S, dP;
    u32x4 ef[2];
    static_for<PD>([&](auto ff) __attribute__((always_inline)) { issue(ff, kt, vt); });
    __builtin_amdgcn_sched_barrier(0);
    static_for<NFT>([&](auto ff) __attribute__((always_inline)) {
      constexpr int F = decltype(ff)::value, kb = F / NFB, f = F % NFB, slot = F % PD;
      if constexpr (f < KS) {
        if constexpr (f == 0) {
#pragma unroll
          for (int i = 0; i < 16; ++i) S[i] = 0.f;
        }
        S = mfma(ring[slot], qf[f], S);
      } else if constexpr (f < 2 * KS) {
        constexpr int ks = f - KS;
        if constexpr (ks == 0) {
#pragma unroll
          for (int i = 0; i < 16; ++i) dP[i] = 0.f;
        }
        dP = mfma(ring[slot], dof[ks], dP);
        constexpr int per = 16 / KS;
#pragma unroll
        for (int i = ks * per; i < (ks + 1) * per; ++i) S[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[i], c, nl2));
        if constexpr (ks == KS - 1) {
          if (need_mask) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
              const i32x4 tk = *reinterpret_cast<const i32x4*>(&s_tok[stage][32 * kb + 8 * i4 + 4 * h]);
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (tk[e] > q_pos) S[4 * i4 + e] = 0.f;
            }
          }
        }
      } else {
        constexpr int j = (f - 2 * KS) / DB, db = (f - 2 * KS) % DB;
        if constexpr (db == 0) {          // ds^T of the 16 keys of group j (registers 8 j .. 8 j + 7), packed to bf16
          float ds[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) ds[e] = S[8 * j + e] * (dP[8 * j + e] + nd);
          ef[j] = u32x4{pack2(ds[0], ds[1]), pack2(ds[2], ds[3]), pack2(ds[4], ds[5]), pack2(ds[6], ds[7])};
        }
        dq[db] = mfma(ring[slot], __builtin_bit_cast(bf16x8, ef[j]), dq[db]);
      }
      if constexpr (F + PD < NFT) issue(std::integral_constant<int, F + PD>{}, kt, vt);
      // the fetch of the next tile, one pass at a time between the matrix instructions
      if constexpr (F % (NFT / C::PASSES) == 1) { if (more) fetch_pass(std::integral_constant<int, F / (NFT / C::PASSES)>{}, t + 1, stage ^ 1); }
      __builtin_amdgcn_sched_barrier(0);
    });
  }
  wait_all_loads();

  // ---- epilogue: dq_acc += scale dq.  A lane owns one query row; per (db, i4) it holds 4
  // consecutive columns and its partner lane (+32) the next 4.
  if (q_valid) {
    float* dst0 = p.dq_acc + qoff + 4 * h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        f32x4* dst = reinterpret_cast<f32x4*>(dst0 + 32 * db + 8 * i4);
        f32x4 val = *dst;
#pragma unroll
        for (int e = 0; e < 4; ++e) val[e] = __builtin_fmaf(dq[db][4 * i4 + e], p.scale, val[e]);
        *dst = val;
      }
  }
}

// ------------------------------------------------------------------------------------------------
// dk / dv kernel
// ------------------------------------------------------------------------------------------------
// NW wavefronts of 32 keys each.  The K rows of a wavefront's keys stay in registers; with VLDS the
// V rows stay in LDS instead (read as B operand when needed), which is what lets a wavefront with
// two 32 x D accumulators fit the 256 registers of two wavefronts per SIMD at D = 128.  At D = 64
// the kernel fits 168 registers, i.e. three workgroups of four wavefronts per CU (-6 % against two).
// With SPLIT a workgroup serves one query head of the group only and leaves fp32 partial sums.
// -lse / scale and -delta of a tile's queries come from the arrays the delta kernel left (p.nlse,
// p.ndelta), gathered straight into LDS like the tile itself (no wavefront ever waits on them);
// they are what the score and dout.v accumulators start from.
template <int D, int NW, bool VLDS, bool SPLIT>
__global__ __launch_bounds__(64 * NW, NW == 8 ? 1 : 3) void bwd_dkv_kernel(const BwdLaunch p) {
  using C = BCfg<D, NW>;
  constexpr int KS = D / 16, DB = D / 32, BS = C::BS, NTHREADS = C::NTHREADS;
  constexpr int VST_BYTES = VLDS ? BS * D * 2 : 0;        // stationary V rows, same row layout as a tile
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * C::STAGE_BYTES + VST_BYTES];   // stage: Q tile, dout tile
  __shared__ __attribute__((aligned(256))) float s_nl[2][BT];   // -lse / scale of the tile's queries (-inf: row contributes nothing)
  __shared__ __attribute__((aligned(256))) float s_nd[2][BT];   // -delta of the tile's queries
  __shared__ int s_tmin, s_tmax;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, lq = lane & 31;

  // ---- which (sequence, KV head, key tile)
  const int G = p.Hq / p.Hkv;
  const int total_keys = p.rng_vbeg[p.n_rng];
  const int ktiles = (total_keys + BS - 1) / BS;
  const int w_all = xcd_balanced(blockIdx.x, p.batch * p.Hkv, ktiles * (SPLIT ? G : 1));
  if (w_all < 0) return;
  // Split by head, the work list of a KV head is head-major: the workgroups an XCD runs at one time
  // then stream the query tiles of the same head through its L2, as they do without the split
  // (tile-major measured 9 % slower), and each head's tiles still come by falling work.
  const int per_tile = SPLIT ? G : 1;          // workgroups per key tile
  const int bi = w_all / (ktiles * p.Hkv * per_tile);
  const int w = w_all - bi * (ktiles * p.Hkv * per_tile);
  const int g = w / (ktiles * per_tile);
  const int wt = w - g * (ktiles * per_tile);
  const int v0 = (wt % ktiles) * BS;           // first key of the tile in the virtual concatenation
  const int hh_beg = SPLIT ? wt / ktiles : 0, hh_end = SPLIT ? hh_beg + 1 : G;   // query heads of the group served here

  // smallest global position among the keys of the tile: queries before it see none of them
  if (tid == 0) {
    int tmin = INT_MAX, tmax = -1;
    for (int j = 0; j < p.n_rng; ++j) {
      const int a = max(v0, p.rng_vbeg[j]), b = min(v0 + BS, p.rng_vbeg[j + 1]);
      if (a < b) {
        tmin = min(tmin, p.rng_start[j] + (a - p.rng_vbeg[j]));
        tmax = max(tmax, p.rng_start[j] + (b - 1 - p.rng_vbeg[j]));
      }
    }
    s_tmin = tmin;
    s_tmax = tmax;
  }

  // ---- stationary side: this lane's key (column lq of the wave's strip)
  auto token_of = [&](int vi) __attribute__((always_inline)) {     // global position of virtual key vi (INT_MAX: past the end)
    int tok = INT_MAX;
    for (int j = 0; j < p.n_rng; ++j)
      if (vi >= p.rng_vbeg[j] && vi < p.rng_vbeg[j + 1]) tok = p.rng_start[j] + (vi - p.rng_vbeg[j]);
    return tok;
  };
  const int key_tok = token_of(v0 + wave * 32 + lq);
  const bool key_valid = key_tok != INT_MAX;
  const int64_t koff = bi * p.kv_bstride + (static_cast<int64_t>(key_valid ? key_tok : p.rng_start[0]) * p.Hkv + g) * D;
  bf16x8 kf[KS], vf[VLDS ? 1 : KS];
  {
    const __bf16* ks_ = static_cast<const __bf16*>(p.k) + koff + 8 * h;
    const __bf16* vs_ = static_cast<const __bf16*>(p.v) + koff + 8 * h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(ks_ + 16 * ks);
      if constexpr (!VLDS) vf[ks] = *reinterpret_cast<const bf16x8*>(vs_ + 16 * ks);
    }
  }
  const float c = p.scale * kLog2e;
  // The compiler cannot see the hand-written waits on the tile fetches; left alone it would wait
  // for these loads again inside the loop, before every instruction that reads them, and those
  // waits would then really wait, for the fetch of the next tile.  Using the values here ends that.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    asm volatile("" : "+v"(kf[ks]));
    if constexpr (!VLDS) asm volatile("" : "+v"(vf[ks]));
  }
  __syncthreads();
  const int tmin = s_tmin;
  // the element-wise mask is needed for tiles with a query before the last key of the workgroup,
  // and everywhere if the workgroup holds padding keys
  const int tmax = (v0 + BS > total_keys) ? INT_MAX : (p.causal ? s_tmax : -1);

  // ---- the streamed side: the 64-row tiles of every query block that hold a row at or after tmin,
  // for every query head served here.  The walk goes BACKWARDS over the tiles, from the last tile of
  // the last block down, with the heads innermost: what a workgroup needs is then a prefix of one
  // sequence that is the same for all workgroups of a KV head, so the workgroups an XCD runs
  // together read the same tile at the same time and it comes from HBM once for all of them.  (Walked
  // forwards, or with the heads outermost, each workgroup is somewhere else in the stream: the launch
  // of the rank's own keys then fetched 9.9 GB instead of about 1.)  Iteration state (head, block, tile).
  auto first_tile = [&](int blk) __attribute__((always_inline)) {
    return p.causal ? max(0, (tmin - p.blk[blk].pos0) / BT) : 0;
  };
  auto tiles_of = [&](int blk) __attribute__((always_inline)) { return (p.blk[blk].n + BT - 1) / BT; };
  struct It { int hh, blk, qt; };
  // the first state at or after (hh, blk, qt) in walking order that has work; blk < 0 means done
  auto settle = [&](It it) __attribute__((always_inline)) {
    if (it.hh >= hh_end) { it.hh = hh_beg; --it.qt; }
    while (it.blk >= 0) {
      if (it.qt >= first_tile(it.blk)) return it;
      --it.blk;
      if (it.blk >= 0) it.qt = tiles_of(it.blk) - 1;
    }
    return it;
  };

  const int fr = tid / C::UNITS, fu = tid % C::UNITS;
  const unsigned col = C::swz(fr, fu) * 16;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned char* Qg = static_cast<const unsigned char*>(p.q) + bi * p.q_bstride * 2;
  const unsigned char* Og = static_cast<const unsigned char*>(p.dout) + bi * p.q_bstride * 2;
  const unsigned q_row_bytes = static_cast<unsigned>(p.Hq) * D * 2;
  // The fetch of a tile comes in pieces (pass i = the Q and dout rows fr + RPP i; lse and delta of
  // the tile's queries with the last one, by the first wavefront: rows past the end of the block
  // take the entry behind the last row, -inf and 0) that the loop drops between its matrix
  // instructions: a burst of direct loads stalls the issuing wavefront once its queue is full.
  const int64_t n_rows_all = static_cast<int64_t>(p.batch) * p.lse_bstride;
  const unsigned char* L2g = reinterpret_cast<const unsigned char*>(p.nlse + bi * p.lse_bstride);
  const unsigned char* Dlg = reinterpret_cast<const unsigned char*>(p.ndelta + bi * p.lse_bstride);
  const unsigned past_end = static_cast<unsigned>(n_rows_all - bi * p.lse_bstride) * 4;
  static_assert(C::PASSES == 2, "the loop places two fetch pieces per tile");
  auto fetch_pass = [&](auto ii, const It& it, int stage) __attribute__((always_inline)) {
    constexpr int i = decltype(ii)::value;
    const BwdBlock& B = p.blk[it.blk];
    const int hq = g * G + it.hh;
    unsigned char* dst = smem + stage * C::STAGE_BYTES + wave_u * 1024;
    {
      const int r = min(it.qt * BT + fr + C::RPP * i, B.n - 1);      // rows past the end repeat the last one and are switched off below
      const unsigned off = static_cast<unsigned>(B.row0 + r) * q_row_bytes + static_cast<unsigned>(hq) * D * 2 + col;
      dma16(Qg, off, dst + i * NTHREADS * 16);
      dma16(Og, off, dst + C::TILE_BYTES + i * NTHREADS * 16);
    }
    if constexpr (i == C::PASSES - 1) if (wave_u == 0) {
      // the lane number, formed here: held in a register across the loop it is one register too many
      int zero = 0;
      asm volatile("" : "+v"(zero));
      const int lane_now = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, zero));
      const int r = it.qt * BT + lane_now;
      const unsigned off = r < B.n ? static_cast<unsigned>((B.row0 + r) * p.Hq + hq) * 4 : past_end;
      global_to_lds_4<true>(L2g, off, reinterpret_cast<unsigned char*>(&s_nl[stage][0]));
      global_to_lds_4<true>(Dlg, off, reinterpret_cast<unsigned char*>(&s_nd[stage][0]));
    }
  };
  auto fetch = [&](const It& it, int stage) __attribute__((always_inline)) {
    static_for<C::PASSES>([&](auto ii) __attribute__((always_inline)) { fetch_pass(ii, it, stage); });
  };

  ReadAddr<D> ra;
  ra.init(lane);

  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dk[db][i] = 0.f; dv[db][i] = 0.f; }

  // the V rows of the workgroup's keys, laid out like a tile (rows past the end repeat a valid row)
  if constexpr (VLDS) {
    const unsigned char* Vg = static_cast<const unsigned char*>(p.v) + (bi * p.kv_bstride + static_cast<int64_t>(g) * D) * 2;
    const unsigned kv_row_bytes = static_cast<unsigned>(p.Hkv) * D * 2;
    unsigned char* dst = smem + 2 * C::STAGE_BYTES + wave_u * 1024;
#pragma unroll
    for (int i = 0; i < BS / C::RPP; ++i) {
      const int tok = token_of(v0 + fr + C::RPP * i);
      const unsigned off = static_cast<unsigned>(tok == INT_MAX ? p.rng_start[0] : tok) * kv_row_bytes + col;
      dma16(Vg, off, dst + i * NTHREADS * 16);
    }
  }

  // The matrix instructions of a tile take their A operands (and with VLDS the V rows, a B operand)
  // as one stream of fragments read PD ahead.  A lane's fragment addresses differ from its first one
  // of the kind only in the swizzled unit number, i.e. by an XOR with a constant below the row
  // pitch (32 ks for row fragments, 64 db for transposed ones), so three or four address registers
  // serve the whole tile: the vector instruction per read is cheap here, 24 registers are not.
  // The empty asm statements make the compiler form each address where it is used instead of
  // keeping all of them.
  constexpr int NFB = 2 * KS + 4 * DB, NFT = 2 * NFB, PD = VLDS ? 3 : 2;
  static_assert(32 * (KS - 1) < D * 2 && 64 * (DB - 1) < D * 2, "the XOR must stay inside a row");
  bf16x8 ring[PD];                 // fragments in flight (slot = fragment % PD)
  bf16x8 vring[VLDS ? PD : 1];
  unsigned a_row = 0, a_tr0 = 0, a_tr1 = 0, a_v = 0;   // byte offsets in smem of this lane's first fragments (current stage; V rows)
  auto issue = [&](auto ff) __attribute__((always_inline)) {
    constexpr int F = decltype(ff)::value, qb = F / NFB, f = F % NFB, slot = F % PD;
    unsigned& av_ = a_v;
    bf16x8* vr_ = vring;
    if constexpr (f < KS) {
      ring[slot] = lds_row8(smem + (a_row ^ (32u * f)) + qb * 32 * D * 2);
    } else if constexpr (f < 2 * KS) {
      constexpr int ks = f - KS;
      ring[slot] = lds_row8(smem + (a_row ^ (32u * ks)) + qb * 32 * D * 2 + C::TILE_BYTES);
      if constexpr (VLDS) vr_[slot] = lds_row8(smem + (av_ ^ (32u * ks)));
    } else if constexpr (f < 2 * KS + 2 * DB) {
      constexpr int j = (f - 2 * KS) / DB, db = (f - 2 * KS) % DB, grp = (2 * qb + j) * 16 * D * 2 + C::TILE_BYTES;
      ring[slot] = lds_tr8(smem + (a_tr0 ^ (64u * db)) + grp, smem + (a_tr1 ^ (64u * db)) + grp);
    } else {
      constexpr int j = (f - 2 * KS - 2 * DB) / DB, db = (f - 2 * KS - 2 * DB) % DB, grp = (2 * qb + j) * 16 * D * 2;
      ring[slot] = lds_tr8(smem + (a_tr0 ^ (64u * db)) + grp, smem + (a_tr1 ^ (64u * db)) + grp);
    }
    if constexpr (f == KS - 1 || f == 2 * KS - 1 || f == 2 * KS + 2 * DB - 1 || f == NFB - 1)
      asm volatile("" : "+v"(a_row), "+v"(a_tr0), "+v"(a_tr1), "+v"(av_));
  };

  It cur = settle(It{hh_beg, p.n_blk - 1, tiles_of(p.n_blk - 1) - 1});
  if (cur.blk >= 0) fetch(cur, 0);
  int stage = 0;
  while (cur.blk >= 0) {
    const It nxt = settle(It{cur.hh + 1, cur.blk, cur.qt});
    wait_all_loads();
    __syncthreads();                 // the current tile is complete; nobody reads the other stage any more
    const bool more = nxt.blk >= 0;
    if (more) fetch_pass(std::integral_constant<int, 0>{}, nxt, stage ^ 1);
    const int pos0 = p.causal ? p.blk[cur.blk].pos0 + cur.qt * BT : 0;
    const bool need_mask = tmax > pos0;
    {
      // The matrix instructions of a tile as one stream of operand fragments, per 32-query block qb:
      // KS row fragments of Q (scores S), KS row fragments of dout (and of V: dP = dout.v), 2 DB
      // transposed fragments of dout (dv), 2 DB transposed fragments of Q (dk).  The reads of
      // fragment F + PD are issued right after the instruction that consumed fragment F.
      // S starts from -lse / scale and dP from -delta of the row (register 4 i4 + e belongs to query
      // 8 i4 + 4 h + e of the block: four 16-byte reads each, issued a phase ahead, while the
      // registers are free), so p = exp2(c S) and ds = p dP are one and two instructions per value.
      // That vector work rides in the shadow of matrix instructions that do not need it: p of
      // 16 / KS queries beside each dP instruction, ds of 16 / (2 DB) queries beside each dv
      // instruction.  p and ds go to bf16 pairs as they are formed (word v / 2 = values v, v + 1;
      // words 4 j .. 4 j + 3 are the B operand of query group j).  Scheduling barriers keep the order.
      constexpr int VPS = 16 / KS, VPD = 16 / (2 * DB);
      static_assert(VPS % 2 == 0 && VPD % 2 == 0, "values are packed in pairs");
      f32x16 S, dP;
      unsigned pw[8], ew[8];
      auto start_from = [&](f32x16& acc, const float* rows, int qb) __attribute__((always_inline)) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const f32x4 t = *reinterpret_cast<const f32x4*>(rows + 32 * qb + 8 * i4 + 4 * h);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[4 * i4 + e] = t[e];
        }
      };
      a_row = stage * C::STAGE_BYTES + ra.row[0];
      a_tr0 = stage * C::STAGE_BYTES + ra.tr[0][0];
      a_tr1 = stage * C::STAGE_BYTES + ra.tr[0][1];
      a_v = 2 * C::STAGE_BYTES + wave * 32 * D * 2 + ra.row[0];
      asm volatile("" : "+v"(a_row), "+v"(a_tr0), "+v"(a_tr1), "+v"(a_v));
      start_from(S, &s_nl[stage][0], 0);
      static_for<PD>([&](auto ff) __attribute__((always_inline)) { issue(ff); });
      __builtin_amdgcn_sched_barrier(0);
      static_for<NFT>([&](auto ff) __attribute__((always_inline)) {
        constexpr int F = decltype(ff)::value, qb = F / NFB, f = F % NFB, slot = F % PD;
        // With one workgroup per CU the two wavefronts of a SIMD belong to it and leave the tile's
        // barrier together; the arbiter then favours the older one all tile long and the younger
        // finishes a fifth later.  The younger one goes first in the first query block (-1.7 %).
        if constexpr (VLDS && f == 0) {
          if (wave_u >= NW / 2) { if constexpr (qb == 0) asm volatile("s_setprio 1"); else asm volatile("s_setprio 0"); }
        }
        if constexpr (f < KS) {
          S = mfma(ring[slot], kf[f], S);
          if constexpr (f == 0) start_from(dP, &s_nd[stage][0], qb);
        } else if constexpr (f < 2 * KS) {
          constexpr int ks = f - KS, u0 = ks * VPS;
          if constexpr (VLDS) dP = mfma(ring[slot], vring[slot], dP);
          else dP = mfma(ring[slot], vf[ks], dP);
#pragma unroll
          for (int e = 0; e < VPS; ++e) S[u0 + e] = __builtin_amdgcn_exp2f(S[u0 + e] * c);
          if (need_mask) {
#pragma unroll
            for (int e = 0; e < VPS; ++e) {
              const int q_pos = p.causal ? pos0 + 32 * qb + 8 * ((u0 + e) / 4) + 4 * h + (u0 + e) % 4 : INT_MAX - 1;
              if (key_tok > q_pos) S[u0 + e] = 0.f;
            }
          }
#pragma unroll
          for (int e = 0; e < VPS; e += 2) pw[(u0 + e) / 2] = pack2(S[u0 + e], S[u0 + e + 1]);
        } else if constexpr (f < 2 * KS + 2 * DB) {
          constexpr int i = f - 2 * KS, j = i / DB, db = i % DB, u0 = i * VPD;
          const u32x4 pf = {pw[4 * j], pw[4 * j + 1], pw[4 * j + 2], pw[4 * j + 3]};
          dv[db] = mfma(ring[slot], __builtin_bit_cast(bf16x8, pf), dv[db]);
#pragma unroll
          for (int e = 0; e < VPD; e += 2)
            ew[(u0 + e) / 2] = pack2(S[u0 + e] * dP[u0 + e], S[u0 + e + 1] * dP[u0 + e + 1]);
        } else {
          constexpr int j = (f - 2 * KS - 2 * DB) / DB, db = (f - 2 * KS - 2 * DB) % DB;
          const u32x4 ef = {ew[4 * j], ew[4 * j + 1], ew[4 * j + 2], ew[4 * j + 3]};
          dk[db] = mfma(ring[slot], __builtin_bit_cast(bf16x8, ef), dk[db]);
          // the next block's scores start from its rows' values; S is free from here on
          if constexpr (f == 2 * KS + 2 * DB && qb == 0) start_from(S, &s_nl[stage][0], 1);
        }
        if constexpr (F + PD < NFT) issue(std::integral_constant<int, F + PD>{});
        if constexpr (F == NFT / 2) { if (more) fetch_pass(std::integral_constant<int, 1>{}, nxt, stage ^ 1); }
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    cur = nxt;
    stage ^= 1;
  }
  wait_all_loads();

  // ---- epilogue: a lane owns one key row; per (db, i4) it holds 4 consecutive columns
  if constexpr (SPLIT) {
    if (key_valid) {
      const int64_t vi = v0 + wave * 32 + lq;
      const int64_t poff = (((static_cast<int64_t>(bi) * G + hh_beg) * total_keys + vi) * p.Hkv + g) * D + 4 * h;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const f32x4 a = {dk[db][4 * i4], dk[db][4 * i4 + 1], dk[db][4 * i4 + 2], dk[db][4 * i4 + 3]};
          const f32x4 b = {dv[db][4 * i4], dv[db][4 * i4 + 1], dv[db][4 * i4 + 2], dv[db][4 * i4 + 3]};
          *reinterpret_cast<f32x4*>(p.part_dk + poff + 32 * db + 8 * i4) = a;
          *reinterpret_cast<f32x4*>(p.part_dv + poff + 32 * db + 8 * i4) = b;
        }
    }
    return;
  }
  if (key_valid) {
    __bf16* dkp = static_cast<__bf16*>(p.dk) + koff + 4 * h;
    __bf16* dvp = static_cast<__bf16*>(p.dv) + koff + 4 * h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        bf16x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[e] = static_cast<__bf16>(dk[db][4 * i4 + e] * p.scale);
          b[e] = static_cast<__bf16>(dv[db][4 * i4 + e]);
        }
        *reinterpret_cast<bf16x4*>(dkp + 32 * db + 8 * i4) = a;
        *reinterpret_cast<bf16x4*>(dvp + 32 * db + 8 * i4) = b;
      }
  }
}

// ------------------------------------------------------------------------------------------------
// delta = sum_d dout * out per (row, head); D / 8 lanes per row.  Written as -delta, and beside it
// -lse / scale (-inf for a row that saw no key): what the dq and dk/dv kernels start their dout.v
// and score accumulators from.  Behind the last row of both arrays sits the entry for "no such
// row": 0 and -inf.
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                                                        const float* __restrict__ lse, float* __restrict__ ndelta,
                                                        float* __restrict__ nlse, float scale, int64_t n_rows) {
  constexpr int LPR = D / 8;                    // lanes per (row, head)
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int64_t row = idx / LPR;
  const int part = static_cast<int>(idx % LPR);
  float s = 0.f;
  if (row < n_rows) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(out + row * D + 8 * part);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(dout + row * D + 8 * part);
#pragma unroll
    for (int e = 0; e < 8; ++e) s = __builtin_fmaf(static_cast<float>(a[e]), static_cast<float>(b[e]), s);
  }
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
  if (row < n_rows && part == 0) {
    ndelta[row] = -s;
    const float l = lse[row];
    nlse[row] = l > -__builtin_inff() ? -l / scale : -__builtin_inff();
  }
  if (idx == 0) {
    ndelta[n_rows] = 0.f;
    nlse[n_rows] = -__builtin_inff();
  }
}

// dk, dv of a launch split by query head: one thread per (sequence, key, KV head, 4 columns) adds the
// G partial sums in the order of the heads, so the result does not depend on how the launch ran.
template <int D>
__global__ __launch_bounds__(256) void bwd_dkv_reduce_kernel(const BwdLaunch p) {
  constexpr int C4 = D / 4;
  const int total_keys = p.rng_vbeg[p.n_rng];
  const int G = p.Hq / p.Hkv;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const int64_t per_b = static_cast<int64_t>(total_keys) * p.Hkv * C4;
  if (idx >= per_b * p.batch) return;
  const int64_t bi = idx / per_b;
  const int64_t r = idx - bi * per_b;
  const int c4 = static_cast<int>(r % C4);
  const int g = static_cast<int>((r / C4) % p.Hkv);
  const int vi = static_cast<int>(r / (static_cast<int64_t>(C4) * p.Hkv));
  int tok = 0;
  for (int j = 0; j < p.n_rng; ++j)
    if (vi >= p.rng_vbeg[j] && vi < p.rng_vbeg[j + 1]) tok = p.rng_start[j] + (vi - p.rng_vbeg[j]);
  f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
  for (int hh = 0; hh < G; ++hh) {
    const int64_t poff = ((((bi * G + hh) * total_keys + vi) * p.Hkv + g) * C4 + c4) * 4;
    const f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p.part_dk + poff));
    const f32x4 y = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p.part_dv + poff));
#pragma unroll
    for (int e = 0; e < 4; ++e) { a[e] += x[e]; b[e] += y[e]; }
  }
  bf16x4 ka, vb;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    ka[e] = static_cast<__bf16>(a[e] * p.scale);
    vb[e] = static_cast<__bf16>(b[e]);
  }
  const int64_t koff = bi * p.kv_bstride + (static_cast<int64_t>(tok) * p.Hkv + g) * D + 4 * c4;
  *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.dk) + koff) = ka;
  *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.dv) + koff) = vb;
}

__global__ __launch_bounds__(256) void bwd_zero_kernel(f32x4* __restrict__ dst, int64_t n4) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n4) dst[i] = f32x4{0.f, 0.f, 0.f, 0.f};
}

}  // namespace

hipError_t launch_bwd_dq_bf16(const BwdLaunch& p, int d, hipStream_t stream) {
  int64_t tiles = 0;
  constexpr int BS = 128;
  for (int t = 0; t < p.n_tasks; ++t) tiles += (p.task[t].n_q + BS - 1) / BS;
  const int64_t items = tiles * p.Hq * p.batch;
  if (items == 0) return hipSuccess;
  if (items > INT_MAX) return hipErrorInvalidValue;
  const int64_t units = static_cast<int64_t>(p.batch) * p.Hkv;
  const int64_t blocks = xcd_balanced_blocks(units, items / units);
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  if (d == 128) return TASP_LAUNCH((bwd_dq_kernel<128>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, p);
  if (d == 64) return TASP_LAUNCH((bwd_dq_kernel<64>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, p);
  return hipErrorInvalidValue;
}

template <int D, int NW, bool VLDS>
hipError_t launch_dkv_variant(const BwdLaunch& p, hipStream_t stream) {
  constexpr int BS = 32 * NW;
  const int64_t total = p.rng_vbeg[p.n_rng];
  const int64_t items = (total + BS - 1) / BS * p.Hkv * p.batch * (p.split_heads ? p.Hq / p.Hkv : 1);
  if (items == 0) return hipSuccess;
  if (items > INT_MAX) return hipErrorInvalidValue;
  const int64_t units = static_cast<int64_t>(p.batch) * p.Hkv;
  const int64_t blocks = xcd_balanced_blocks(units, items / units);
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(blocks)), block(64 * NW);
  if (p.split_heads) return TASP_LAUNCH((bwd_dkv_kernel<D, NW, VLDS, true>), grid, block, stream, p);
  return TASP_LAUNCH((bwd_dkv_kernel<D, NW, VLDS, false>), grid, block, stream, p);
}

hipError_t launch_bwd_dkv_bf16(const BwdLaunch& p, int d, hipStream_t stream) {
  if (d == 128) return launch_dkv_variant<128, 8, true>(p, stream);
  if (d == 64) return launch_dkv_variant<64, 4, false>(p, stream);
  return hipErrorInvalidValue;
}

int64_t bwd_dkv_workgroups(const BwdLaunch& p, int d) {
  const int bs = d == 128 ? 256 : 128;
  return (static_cast<int64_t>(p.rng_vbeg[p.n_rng]) + bs - 1) / bs * p.Hkv * p.batch;
}

int bwd_dkv_resident_workgroups(int d) {
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    cus = 256;
  return cus * (d == 128 ? 1 : 3);
}

hipError_t launch_bwd_dkv_reduce(const BwdLaunch& p, int d, hipStream_t stream) {
  const int64_t threads = static_cast<int64_t>(p.rng_vbeg[p.n_rng]) * p.Hkv * (d / 4) * p.batch;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks == 0) return hipSuccess;
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  if (d == 128) return TASP_LAUNCH((bwd_dkv_reduce_kernel<128>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, p);
  if (d == 64) return TASP_LAUNCH((bwd_dkv_reduce_kernel<64>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, p);
  return hipErrorInvalidValue;
}

hipError_t launch_bwd_delta_bf16(const void* out, const void* dout, const float* lse, float* ndelta, float* nlse,
                                 float scale, int64_t n_rows, int d, hipStream_t stream) {
  if (n_rows == 0) return hipSuccess;
  const int64_t threads = n_rows * (d / 8);
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  const __bf16* o = static_cast<const __bf16*>(out);
  const __bf16* g = static_cast<const __bf16*>(dout);
  if (d == 128) return TASP_LAUNCH((bwd_delta_kernel<128>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, o, g, lse, ndelta, nlse, scale, n_rows);
  if (d == 64) return TASP_LAUNCH((bwd_delta_kernel<64>), dim3(static_cast<unsigned>(blocks)), dim3(256), stream, o, g, lse, ndelta, nlse, scale, n_rows);
  return hipErrorInvalidValue;
}

hipError_t launch_zero_f32(float* dst, int64_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  if (n % 4 != 0) return hipErrorInvalidValue;
  const int64_t blocks = (n / 4 + 255) / 256;
  if (blocks > INT_MAX) return hipErrorInvalidValue;
  return TASP_LAUNCH(bwd_zero_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), stream,
                     reinterpret_cast<f32x4*>(dst), n / 4);
}

}  // namespace tasp
