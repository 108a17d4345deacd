/*
 * tasp.h -- C ABI of the single-GPU hot path of TASP (topology-aware sequence parallelism,
 * arXiv 2509.26541) for AMD MI355X (gfx950).
 *
 * One process drives one GPU and plays one "virtual rank" r of an N-rank sequence-parallel group:
 * the GPU holds the whole K and V of the sequence and rank r's local queries, and performs rank r's
 * share of the forward pass of Algorithm 3 -- N steps; at step s the rank attends to the N-1 KV
 * sub-chunks that the Multi-Ring AllGather (Sec. 3.2.2) would have delivered to it at that step,
 * concatenated in ring order, and folds the partial (output, lse) into a running pair.  The
 * transport itself (AlltoAll between GPUs) is not part of this library.
 *
 * Conventions
 *   - Every function returns TASP_OK (0) or a negative tasp_status.  Nothing throws, aborts or prints.
 *   - "host" / "device" is stated for every pointer.  The library never allocates device memory;
 *     device work is enqueued on the caller's HIP stream and is asynchronous.  Its only state
 *     outside the objects it hands out: per thread, the last HIP error it met (tasp_last_hip_error),
 *     and per GPU the fixed scratch array of tasp_chunk_attn_static.
 *   - Tensors are dense, row-major, with the last index fastest.
 *   - Token positions are global positions in [0, S).
 */
#ifndef TASP_H
#define TASP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tasp_status {
  TASP_OK = 0,
  TASP_EINVAL = -1,            /* null pointer, N < 2, rank outside [0,N), S not divisible, Hq % Hkv != 0 ... */
  TASP_EUNSUPPORTED_N = -2,    /* N for which no ring decomposition is implemented (see tasp_schedule_create) */
  TASP_EUNSUPPORTED_SHAPE = -3,/* head dim / dtype / size outside what the kernels cover */
  TASP_EALIGN = -4,            /* a device pointer is not 16-byte aligned */
  TASP_EWORKSPACE = -5,        /* workspace missing or smaller than tasp_chunk_attn_workspace_bytes() */
  TASP_EHIP = -6,              /* a HIP call or kernel launch failed */
  TASP_ENOMEM = -7             /* host allocation failed */
} tasp_status;

enum { TASP_MASK_FULL = 0, TASP_MASK_ZIGZAG_CAUSAL = 1 };
enum { TASP_DTYPE_FP32 = 0, TASP_DTYPE_BF16 = 1 };
enum { TASP_ORDER_TASP = 0, TASP_ORDER_RING = 1 };

/* Human-readable text for a status code (static storage, never NULL). */
const char* tasp_strerror(int status);
/* After TASP_EHIP: the HIP runtime's text for the last HIP error the calling thread met inside this
 * library ("no error" if none so far).  Static storage owned by the HIP runtime. */
const char* tasp_last_hip_error(void);

/* ------------------------------------------------------------------------------------------------
 * tasp_schedule(N, rank): ring decomposition, routing tables and arrival order.      [host only]
 *
 * Sec. 3.1.2, Algorithm 1: the complete directed graph K_N is decomposed into N-1 arc-disjoint
 * directed Hamiltonian cycles ("orthogonal ring datapaths", Sec. 3.1.1 eq. (2)).  Algorithm 1 is
 * defined for N >= 8 with N % 4 == 0.  N == 4 has no such decomposition; three Hamiltonian rings
 * with the least possible overlap are used ([0,1,2,3] [0,1,3,2] [0,2,3,1]) and
 * tasp_schedule_max_arc_load() reports 2 instead of 1.  Any other N gives TASP_EUNSUPPORTED_N.
 *
 * The object is immutable, lives in host memory and is owned by the library until
 * tasp_schedule_destroy().  All array accessors return host pointers into it.
 * ---------------------------------------------------------------------------------------------- */
typedef struct tasp_schedule tasp_schedule_t;

int  tasp_schedule_create(int32_t n_ranks, int32_t rank, tasp_schedule_t** out);
void tasp_schedule_destroy(tasp_schedule_t* s);

/* Sec. 3.1.3, the (m-K_m-m)^u-decomposition for u nodes of m ranks each (N = m*u; the ranks of node
 * c are c*m .. c*m+m-1): the complete graph of every node is cut into m Hamiltonian paths (the
 * row-complete Latin square of the zig-zag sequence 0,1,m-1,2,...), and ring i runs through path i
 * of node 0, path i of node 1, ... and closes from the last node to the first.  It has m rings
 * instead of N-1: every arc inside a node lies on exactly one ring, every rank sends to the next
 * node once and receives from the previous node once.  A chunk is cut in m sub-chunks; everything
 * else (tables, ranges, tasp_chunk_attn) works as with tasp_schedule_create.
 * ranks_per_node must be even and n_nodes >= 2 (the closing arcs of a single node would repeat arcs
 * of its paths), N <= 4096; otherwise TASP_EUNSUPPORTED_N (TASP_EINVAL for non-positive arguments
 * or a rank outside [0, N)). */
int  tasp_schedule_create_multinode(int32_t ranks_per_node, int32_t n_nodes, int32_t rank, tasp_schedule_t** out);

int32_t tasp_schedule_n_ranks(const tasp_schedule_t* s);
int32_t tasp_schedule_rank(const tasp_schedule_t* s);
int32_t tasp_schedule_n_rings(const tasp_schedule_t* s);          /* R: N-1, or m for the multi-node scheme */
int32_t tasp_schedule_max_arc_load(const tasp_schedule_t* s);     /* 1: true decomposition, 2: N == 4 */

/* rings[i*N + j], i < R, j < N: rank at position j of ring i; data moves from position j to
 * position (j+1) % N (Algorithm 1's h_cycles, Algorithm 2's looping matrix). */
const int32_t* tasp_schedule_rings(const tasp_schedule_t* s);
/* Algorithm 2.  out_mapping[u*N + v] = ring on which u sends to v; in_mapping[u*N + v] = ring on
 * which u receives from v; -1 on the diagonal and on arcs no ring uses.  For an arc on two rings
 * (N == 4 only) the lower ring id is stored. */
const int32_t* tasp_schedule_out_mapping(const tasp_schedule_t* s);
const int32_t* tasp_schedule_in_mapping(const tasp_schedule_t* s);
/* Sec. 3.2.2, Fig. 4.  arrival[s*R + i] = rank at which the sub-chunk t[i, .] that this rank
 * holds on ring i at step s started; row 0 is the rank itself. */
const int32_t* tasp_schedule_arrival(const tasp_schedule_t* s);

/* Sec. 3.2.3.  Global token ranges [start, end) of sub-chunk t[ring, src_rank]:
 *   TASP_MASK_FULL           one range: piece `ring` of the contiguous chunk of eq. (3);
 *   TASP_MASK_ZIGZAG_CAUSAL  two ranges: piece `ring` of half-chunk src_rank (eq. (5)) and its
 *                            mirror image in half-chunk 2N-1-src_rank (eq. (6)).
 * Piece i of a block of `len` tokens is [i*len/R, (i+1)*len/R) with integer division (R rings).
 * ranges (host, 4 entries) receives start0,end0[,start1,end1]; *n_ranges receives 1 or 2.
 * S must be a positive multiple of N (FULL) or 2N (ZIGZAG_CAUSAL). */
int tasp_subchunk_ranges(const tasp_schedule_t* s, int64_t S, int32_t mask_mode, int32_t ring,
                         int32_t src_rank, int64_t ranges[4], int32_t* n_ranges);

/* The KV segments one block of local query rows attends to at one step, in concatenation order
 * (ring order, Algorithm 3), after dropping what the causal mask hides completely (the load-balance
 * argument of Sec. 3.2.3) and after joining neighbours that are contiguous in the sequence.
 *   q_block  0: all local rows (FULL), or the first half-chunk's rows (ZIGZAG_CAUSAL);
 *            1: the second half-chunk's rows (ZIGZAG_CAUSAL only).
 *   order    TASP_ORDER_TASP: the multi-ring arrival order; TASP_ORDER_RING: plain Ring /
 *            Zig-zag Ring Attention, one whole chunk per step from rank (r - step) mod N.
 * seg (host, 2*cap entries) receives start,end pairs; diag (host, cap entries) is 1 where the
 * segment straddles the causal diagonal of the block (needs an element-wise mask), else 0.
 * *n_seg receives the count; TASP_EINVAL if cap is too small. */
int tasp_step_segments(const tasp_schedule_t* s, int64_t S, int32_t mask_mode, int32_t order,
                       int32_t step, int32_t q_block, int64_t* seg, int32_t* diag, int32_t cap,
                       int32_t* n_seg);

/* ------------------------------------------------------------------------------------------------
 * tasp_chunk_attn: the forward pass of Algorithm 3 for one rank.                  [device work]
 *
 *   q, out   device, [L, Hq, d]   rank-local rows, L = S/N.  ZIGZAG_CAUSAL: local row l < H = S/(2N)
 *                                  is global position r*H + l, row l >= H is S - (r+1)*H + (l-H)
 *                                  (eq. (4)).  FULL: local row l is global r*L + l (eq. (3)).
 *   k, v     device, [S, Hkv, d]  the whole sequence in natural token order; a sub-chunk is a row
 *                                  range of these (the stand-in for the receive buffers of Alg. 3).
 *   lse      device, [L, Hq] fp32 natural-log sum-exp of the scaled scores.
 *   dtype    element type of q, k, v, out (fp32, or bf16 with fp32 accumulation).
 *   Query head h reads KV head h*Hkv/Hq.  Causal: key t is visible to query p iff t <= p.
 *   softmax_scale 0 means 1/sqrt(d).
 *   fuse_merge 0: every step writes a partial (out_s, lse_s) and tasp_lse_merge's kernel folds it in
 *                 (update_out_lse of Algorithm 3);  1: the attention kernel folds it in itself.
 *   workspace device, >= tasp_chunk_attn_workspace_bytes() bytes, 256-byte aligned, caller-owned,
 *             contents undefined on entry and exit.
 *   fuse_steps 0: one attention launch per step, each followed by update_out_lse as above (the
 *                 form in which a step can start as soon as its sub-chunks have arrived);
 *              1: ONE launch walks the sub-chunks of all N steps in arrival order and carries the
 *                 running max / sum / output across them, so no partial pair is ever written or
 *                 merged (the log-sum-exp rescale happens in registers).  For callers whose K and V
 *                 are resident when the call is made; it removes the per-step launch, set-up and
 *                 merge costs, which dominate for short sequences.  At most
 *                 TASP_MAX_FUSED_SEGMENTS visible segments per query block over all steps
 *                 (otherwise TASP_EUNSUPPORTED_SHAPE); fuse_merge is ignored.
 *   batch    B independent sequences handled in one call (0 counts as 1, at most 65535): every
 *            tensor gets a leading dimension, q/out [B, L, Hq, d], k/v [B, S, Hkv, d], lse
 *            [B, L, Hq]; all sequences share S, the schedule and the mask (the shape grid of the
 *            paper's evaluation, Sec. 5.1, has batches of up to 128 sequences).
 * Supported: d in {64, 128}; schedules of at most 32 rings (N <= 33 ranks with tasp_schedule_create;
 * with tasp_schedule_create_multinode up to 32 ranks per node and any N it accepts - a call
 * enqueues N steps); S < 2^31; for bf16 also S < 2^24 and S*Hkv*d*2 <= 2^32 bytes (K and V are
 * addressed with 32-bit offsets; with Hkv = 1, less than 2^32).  All device pointers 16-byte aligned.
 * The call only enqueues work on `hip_stream` (a hipStream_t, NULL = default stream); results are
 * valid once the stream has been synchronised.
 * ---------------------------------------------------------------------------------------------- */
typedef struct tasp_attn_args {
  const void* q;
  const void* k;
  const void* v;
  void*       out;
  float*      lse;
  void*       workspace;
  size_t      workspace_bytes;
  int64_t     S;
  int32_t     Hq, Hkv, d;
  int32_t     dtype;
  int32_t     mask_mode;
  int32_t     order;          /* TASP_ORDER_TASP or TASP_ORDER_RING */
  int32_t     fuse_merge;
  float       softmax_scale;
  int32_t     batch;
  int32_t     fuse_steps;
} tasp_attn_args;
#define TASP_MAX_FUSED_SEGMENTS 1024

size_t tasp_chunk_attn_workspace_bytes(const tasp_schedule_t* s, const tasp_attn_args* a);
int    tasp_chunk_attn(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): tasp_chunk_attn with the workspace taken from a fixed array of
 * TASP_STATIC_SCRATCH_BYTES bytes inside the library's code object instead of from the caller
 * (a->workspace and a->workspace_bytes are ignored).  Each GPU the library runs on holds that array
 * from the time the library is loaded until the process ends.  The call allocates nothing on the
 * device and frees nothing; inputs and outputs are the caller's as before.
 *   - A call whose tasp_chunk_attn_workspace_bytes() exceeds TASP_STATIC_SCRATCH_BYTES returns
 *     TASP_EWORKSPACE and enqueues nothing (bf16: B*L*Hq*d <= 16 Mi elements with fuse_merge, half of
 *     that without; fp32 with fuse_merge needs no workspace at all).
 *   - The device that is current when the call is made must be the device of hip_stream.  The first
 *     call on a device asks the HIP runtime for the array's address on that device (a symbol query;
 *     make that first call outside a stream capture).
 *   - All calls on one GPU share the one array, and it keeps the last call's contents: nothing in it
 *     has to start at zero (step 0 of every call overwrites what it uses), but two calls that overlap
 *     on one GPU (different streams, or different threads) race.  Serialise them.
 * Results are those of tasp_chunk_attn (the same kernels run). */
#define TASP_STATIC_SCRATCH_BYTES (64u << 20)
int tasp_chunk_attn_static(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream);

/* The same call with every kernel launch bracketed by HIP events on `hip_stream`, for measurement.
 * Synchronises the stream before returning.  Times are sums over launches, in milliseconds:
 * attn = step-attention kernels, merge = update_out_lse kernels, other = the final bf16 cast. */
typedef struct tasp_profile {
  double  attn_ms, merge_ms, other_ms;
  int32_t attn_launches, merge_launches, other_launches;
} tasp_profile;
int tasp_chunk_attn_profile(const tasp_schedule_t* s, const tasp_attn_args* a, void* hip_stream,
                            tasp_profile* out);

/* One step of the same pass: the partial (out_s, lse_s) of step `step` alone, before any merge.
 * o_part device [L, Hq, d] fp32, lse_part device [L, Hq] fp32.  Rows that see no key at this step
 * get out = 0, lse = -inf.  a->out, a->lse, a->workspace are not used. */
int tasp_step_attn(const tasp_schedule_t* s, const tasp_attn_args* a, int32_t step,
                   float* o_part, float* lse_part, void* hip_stream);

/* update_out_lse of Algorithm 3, in place on the running pair:
 *   lse' = log(exp(lse_acc) + exp(lse_part))
 *   o'   = exp(lse_acc - lse') * o_acc + exp(lse_part - lse') * o_part
 * o_* device [rows, heads, d] fp32 (16-byte aligned), lse_* device [rows, heads] fp32; d a power of
 * two in [4, 256] (anything else: TASP_EUNSUPPORTED_SHAPE).  A side with
 * lse = -inf contributes nothing; if both are -inf the result is o = 0, lse = -inf. */
int tasp_lse_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                   int64_t rows, int32_t heads, int32_t d, void* hip_stream);

/* All partial pairs of Algorithm 3 merged in one pass instead of N-1 applications of
 * update_out_lse (the fold telescopes to this):
 *   lse = log(sum_i exp(lse_i)),   o = sum_i exp(lse_i - lse) * o_i
 * o_parts / lse_parts: HOST arrays of n_parts DEVICE pointers, o_parts[i] -> [rows, heads, d] fp32
 * (16-byte aligned), lse_parts[i] -> [rows, heads] fp32; they are read during the call only.
 * o_out / lse_out: device, same shapes; they may alias one of the partials (every (row, head) is
 * read completely before it is written).  1 <= n_parts <= TASP_MAX_MERGE_PARTS, d as for
 * tasp_lse_merge.  Partials with lse = -inf contribute nothing; all -inf gives o = 0, lse = -inf.
 * HBM traffic per (row, head): (n_parts + 1)(4d + 4) bytes against 3 (n_parts - 1)(4d + 4) for the fold. */
#define TASP_MAX_MERGE_PARTS 64
int tasp_lse_merge_many(float* o_out, float* lse_out, const float* const* o_parts, const float* const* lse_parts,
                        int32_t n_parts, int64_t rows, int32_t heads, int32_t d, void* hip_stream);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned) by
 * a streaming kernel of this library.  Not part of the method: it gives profilers a transfer of
 * known size with which to scale their HBM traffic counters. */
int tasp_calibration_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Runs `iters` x 32 independent v_mfma_f32_32x32x16_bf16 per wavefront on 2048 workgroups of 8
 * wavefronts (pseudo-random operands of magnitude about one in registers, nothing else in the loop) and stores the number of floating
 * point operations that is in *flops (host pointer, may be NULL).  Not part of the method: timed by
 * the caller it gives the rate the matrix pipe of this GPU sustains at the clock it runs at under
 * load, next to which a fraction of the published peak can be read.  iters in [1, 1 << 20]. */
int tasp_calibration_mfma(int32_t iters, double* flops, void* hip_stream);

/* Issue-cost calibration of the vector issue port of a SIMD.  256 workgroups of eight wavefronts
 * (two per SIMD) repeat `iters` x 4 slots of one v_mfma_f32_32x32x16_bf16 followed by
 *   kind 0: per_slot (8 or 12) v_fma_f32,   kind 1: per_slot (4 or 8) v_exp_f32,
 *   kind 2: eight v_fma_f32 and per_slot (1 or 2) ds_read_b128 (1 KiB of LDS data per wavefront each);
 * cycles_per_slot_x16 (DEVICE pointer, 256 x 8 int64) receives, per workgroup and wavefront, 16 x
 * the shader-clock cycles per slot.  The slowest wavefront of a workgroup gives the time in which
 * its SIMD issued two slots: 2 x (matrix instruction + the rest) port cycles, so two values of
 * per_slot price both terms.  Not part of the method: it is the measurement behind the port-cycle
 * figures with which a caller bounds the attention kernel by vector issue.  iters in [1, 1 << 20];
 * other (kind, per_slot) pairs return TASP_EINVAL. */
int tasp_calibration_issue(int32_t kind, int32_t per_slot, int32_t iters, int64_t* cycles_per_slot_x16,
                           void* hip_stream);

/* Algorithmic work of one tasp_chunk_attn call: 4*d*Hq*(visible (query,key) pairs). */
double tasp_chunk_attn_flops(const tasp_schedule_t* s, const tasp_attn_args* a);

/* ----------------------------------------------------------------------------------------------
 * Backward pass of the same computation.  The paper measures the forward pass only (Sec. 5.1.2);
 * this is the gradient of what tasp_chunk_attn computes, walked in the same arrival order
 * (Algorithm 3): at every step the KV sub-chunks held at that step receive dk and dv from the local
 * query rows (a key is held at exactly one step, so its rows are complete after that step), and dq
 * accumulates over the steps.  The probabilities are recomputed from the final lse:
 *   p = exp(scale q.k - lse),  delta = sum_d dout*out,  ds = p (dout.v - delta),
 *   dq = scale ds k,  dk = scale ds^T q,  dv = p^T dout.
 * dk and dv are THIS RANK'S contribution (its local query rows); with grouped-query attention a KV
 * head receives the sum over its query heads.  In a distributed run they would travel on along the
 * rings with their sub-chunk; that transport is not part of this library.
 *
 * All tensor pointers are DEVICE pointers, 16-byte aligned, dense row-major, laid out as for
 * tasp_chunk_attn: q, out, dout, dq [B, L, Hq, d]; k, v, dk, dv [B, S, Hkv, d]; lse [B, L, Hq] fp32
 * (out and lse as written by tasp_chunk_attn on the same inputs).  dtype is TASP_DTYPE_BF16 (matrix
 * instructions, the measured path) or TASP_DTYPE_FP32 (a plain small-shape path, all arithmetic
 * fp32); d is 64 or 128.  Every row of dq, dk and dv is written.
 * workspace: device, 256-byte aligned, at least tasp_chunk_attn_bwd_workspace_bytes() (the delta
 * vector; for bf16 also lse scaled to base 2 in the same layout, both with one more entry behind the
 * last row, which is why B*L*Hq must stay below 2^30 there (TASP_EUNSUPPORTED_SHAPE otherwise), an
 * fp32 copy of dq and, step by step with Hq > Hkv, fp32 partial dk and dv of
 * one step's keys per query head of a group, twice the size of that copy: a step's dk/dv launch with
 * few, unequal key tiles is cut into one workgroup per key tile and query head, and the partial sums
 * are added in the order of the heads, so results do not depend on timing); contents are scratch.
 * Kernels are enqueued on hip_stream; the call returns without synchronising.  Errors as for
 * tasp_chunk_attn.
 * ---------------------------------------------------------------------------------------------- */
typedef struct tasp_attn_bwd_args {
  const void*  q;
  const void*  k;
  const void*  v;
  const void*  out;
  const float* lse;
  const void*  dout;
  void*        dq;
  void*        dk;
  void*        dv;
  void*        workspace;
  size_t       workspace_bytes;
  int64_t      S;
  int32_t      Hq, Hkv, d;
  int32_t      dtype;
  int32_t      mask_mode;
  int32_t      order;
  float        softmax_scale;   /* 0: 1/sqrt(d) */
  int32_t      batch;           /* 0 counts as 1 */
  void*        aux_stream;      /* optional second HIP stream of the caller (default priority, same device),
                                   or NULL.  The dq and the dk/dv kernels of a step are independent; given a
                                   second stream the dk/dv kernels run there, forked from and joined back
                                   into hip_stream with events, so that each fills the idle compute units at
                                   the other's tail.  Results are identical.  The call must then not be
                                   recorded into a HIP graph. */
  int32_t      fuse_steps;      /* 0: one dq and one dk/dv launch per step; 1: one of each for all steps (as
                                   fuse_steps of tasp_chunk_attn: K, V resident; bf16 only; at most
                                   TASP_MAX_FUSED_SEGMENTS segments per query block) */
} tasp_attn_bwd_args;

size_t tasp_chunk_attn_bwd_workspace_bytes(const tasp_schedule_t* s, const tasp_attn_bwd_args* a);
int    tasp_chunk_attn_bwd(const tasp_schedule_t* s, const tasp_attn_bwd_args* a, void* hip_stream);

/* The same call with every launch bracketed by HIP events; synchronises the stream.  dq = the
 * kernels that accumulate dq, dkv = the kernels that form dk and dv, other = delta and clearing the
 * fp32 dq (one bracket), the final cast, the segment table of fuse_steps, and after every dk/dv
 * launch that was split by query head the launch that adds its partial sums. */
typedef struct tasp_bwd_profile {
  double  dq_ms, dkv_ms, other_ms;
  int32_t dq_launches, dkv_launches, other_launches;
} tasp_bwd_profile;
int tasp_chunk_attn_bwd_profile(const tasp_schedule_t* s, const tasp_attn_bwd_args* a, void* hip_stream,
                                tasp_bwd_profile* out);

/* Algorithmic work of one backward call: five products against the forward's two, i.e. 2.5 times
 * tasp_chunk_attn_flops (the recomputation of the scores in both kernels is not counted). */
double tasp_chunk_attn_bwd_flops(const tasp_schedule_t* s, const tasp_attn_bwd_args* a);

#ifdef __cplusplus
}
#endif
#endif /* TASP_H */
