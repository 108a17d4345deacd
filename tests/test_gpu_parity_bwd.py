"""Parity of the HIP backward pass (through the C ABI) with the fp64 oracle on the same seeded inputs.

Tolerance, bf16: every output element is a sum of products whose factors p and ds are rounded to
bf16 before the matrix instruction (relative 2^-9 each, signs random) and is itself rounded to bf16
once (2^-9 of its value); the bar is  |err| <= 2^-7 |ref| + 2^-8 max|ref|  per tensor, about twice
what the small cases show."""
import numpy as np
import pytest
import torch

from paper_2509_26541_amd import workloads as wl
from tests.helpers import oracle_grads, oracle_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2509_26541_amd import binding
    return binding


def close(name, got, ref):
    got = got.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), name
    err = np.abs(got - ref)
    bound = np.abs(ref) / 128 + np.abs(ref).max() / 256
    worst = float((err / bound).max())
    assert worst <= 1.0, "%s: error %.3f of the bound (max err %.3e, max |ref| %.3e)" % (name, worst, err.max(), np.abs(ref).max())


def forward_backward(tb, w, q, k, v, do, schedule=None, **kw):
    s = tb.tasp_schedule(w.n_ranks, w.rank) if schedule is None else schedule
    qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
    out, lse = tb.tasp_chunk_attn(qd, kd, vd, s, w.mask_mode, fuse_merge=True, **kw)
    dq, dk, dv = tb.tasp_chunk_attn_bwd(qd, kd, vd, out, lse, dod, s, w.mask_mode, **kw)
    torch.cuda.synchronize()
    return dq, dk, dv


SMALL = [
    # name, N, rank, S, Hq, Hkv, d, mask, config whose value recipe is used
    ("zz_n8", 8, 3, 4096, 8, 2, 128, wl.ZIGZAG_CAUSAL, 1),
    ("zz_n8_ragged", 8, 6, 8 * 2 * 100, 4, 2, 128, wl.ZIGZAG_CAUSAL, 1),      # H = 100: ragged query and key tiles
    ("zz_n8_tiny", 8, 0, 112, 2, 1, 128, wl.ZIGZAG_CAUSAL, 1),               # sub-chunks of 1 token
    ("zz_n8_one_row", 8, 5, 16, 2, 2, 128, wl.ZIGZAG_CAUSAL, 1),             # one row per half-chunk, most sub-chunks empty
    ("full_n4_one_row", 4, 3, 4, 2, 1, 64, wl.FULL, 1),                      # L = 1
    ("full_n8", 8, 0, 8 * 331, 4, 4, 128, wl.FULL, 2),                       # L = 331, k scaled by 2
    ("full_n4_gqa4", 4, 2, 4 * 300, 4, 1, 128, wl.FULL, 2),
    ("zz_n16", 16, 5, 16 * 2 * 96, 8, 1, 128, wl.ZIGZAG_CAUSAL, 3),
    ("zz_n8_outliers", 8, 7, 4096, 4, 2, 128, wl.ZIGZAG_CAUSAL, 4),
    ("zz_d64", 8, 2, 4096, 4, 2, 64, wl.ZIGZAG_CAUSAL, 1),
    ("full_d64", 8, 5, 8 * 200, 2, 2, 64, wl.FULL, 2),
    ("zz_d64_mha12", 8, 1, 2048, 12, 12, 64, wl.ZIGZAG_CAUSAL, 1),           # 12 KV heads: pairs of XCDs share three heads
    ("full_gqa_kv3", 8, 4, 8 * 160, 6, 3, 128, wl.FULL, 2),                  # 3 KV heads: all XCDs share them
]


def small_workload(case):
    name, n, rank, S, Hq, Hkv, d, mode, base = case
    b = wl.CONFIGS[base]
    return wl.Workload("bwd_" + name, n, rank, S, Hq, Hkv, d, "bf16", mode, k_scale=b.k_scale,
                       outlier_frac=b.outlier_frac, seed=wl.BASE_SEED + 700 + len(name) + S % 97)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_all_outputs(tb, case):
    """The backward call on its own: out and lse are the oracle's forward results rounded to the
    storage types (bf16, fp32), and the oracle takes delta from that same stored out, so both sides
    see the same inputs."""
    w = small_workload(case)
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    out64, lse64 = oracle_rows(w, q, k, v, range(w.L))
    out = torch.from_numpy(out64).to(torch.bfloat16)
    lse = torch.from_numpy(lse64).to(torch.float32)
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    dq, dk, dv = tb.tasp_chunk_attn_bwd(q.cuda(), k.cuda(), v.cuda(), out.cuda(), lse.cuda(), do.cuda(), s, w.mask_mode)
    torch.cuda.synchronize()
    rq, rk, rv = oracle_grads(w, q, k, v, do, out=out)
    close(w.name + " dq", dq, rq)
    close(w.name + " dk", dk, rk)
    close(w.name + " dv", dv, rv)


# With the outlier recipe one key dominates many rows; there dout.v - delta cancels and the bf16
# rounding of the stored out (an input) decides the result, so the chain is compared where it does not.
CHAIN = [c for c in SMALL if "outliers" not in c[0]]


@pytest.mark.parametrize("case", CHAIN, ids=[c[0] for c in CHAIN])
def test_small_forward_then_backward(tb, case):
    """The two calls in a row as a user makes them (out, lse from tasp_chunk_attn) against the exact gradient."""
    w = small_workload(case)
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    dq, dk, dv = forward_backward(tb, w, q, k, v, do)
    rq, rk, rv = oracle_grads(w, q, k, v, do)
    close(w.name + " dq", dq, rq)
    close(w.name + " dk", dk, rk)
    close(w.name + " dv", dv, rv)


@pytest.mark.parametrize("case", CHAIN, ids=[c[0] for c in CHAIN])
def test_small_single_launch(tb, case):
    """fuse_steps in both passes: one forward launch, then one dq and one dk/dv launch for all steps."""
    w = small_workload(case)
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    dq, dk, dv = forward_backward(tb, w, q, k, v, do, fuse_steps=True)
    rq, rk, rv = oracle_grads(w, q, k, v, do)
    close(w.name + " dq", dq, rq)
    close(w.name + " dk", dk, rk)
    close(w.name + " dv", dv, rv)


def test_ring_order_and_multinode_schedule(tb):
    """The gradient does not depend on the order in which the sub-chunks arrive."""
    w = small_workload(SMALL[1])
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    rq, rk, rv = oracle_grads(w, q, k, v, do)
    dq, dk, dv = forward_backward(tb, w, q, k, v, do, order=tb.ORDER_RING)
    close("ring dq", dq, rq); close("ring dk", dk, rk); close("ring dv", dv, rv)
    dq, dk, dv = forward_backward(tb, w, q, k, v, do, schedule=tb.tasp_schedule_multinode(4, 2, w.rank))
    close("multinode dq", dq, rq); close("multinode dk", dk, rk); close("multinode dv", dv, rv)


def test_batched_equals_separate_calls(tb):
    B = 3
    ws = [wl.Workload("bwd_b%d" % b, 8, 4, 8 * 2 * 72, 4, 2, 128, "bf16", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 800 + 13 * b)
          for b in range(B)]
    data = [wl.make_qkv(w) + (wl.make_dout(w),) for w in ws]
    q, k, v, do = (torch.stack([x[i] for x in data]).cuda() for i in range(4))
    s = tb.tasp_schedule(8, 4)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, wl.ZIGZAG_CAUSAL, fuse_merge=True)
    dq, dk, dv = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, wl.ZIGZAG_CAUSAL)
    torch.cuda.synchronize()
    # the same batch with all steps in one launch and the dk/dv kernel on a second stream
    dq1, dk1, dv1 = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, wl.ZIGZAG_CAUSAL, fuse_steps=True,
                                           aux_stream=torch.cuda.Stream())
    torch.cuda.synchronize()
    for b in range(B):
        rq, rk, rv = oracle_grads(ws[b], *data[b])
        close("b%d dq" % b, dq[b], rq); close("b%d dk" % b, dk[b], rk); close("b%d dv" % b, dv[b], rv)
        close("b%d dq one launch" % b, dq1[b], rq); close("b%d dk one launch" % b, dk1[b], rk)
        close("b%d dv one launch" % b, dv1[b], rv)
        one = tb.tasp_chunk_attn_bwd(q[b].contiguous(), k[b].contiguous(), v[b].contiguous(), out[b].contiguous(),
                                     lse[b].contiguous(), do[b].contiguous(), s, wl.ZIGZAG_CAUSAL)
        torch.cuda.synchronize()
        assert torch.equal(one[0], dq[b]) and torch.equal(one[1], dk[b]) and torch.equal(one[2], dv[b])


def test_second_stream_gives_the_same_bits(tb):
    """dk/dv kernels on a second stream of the caller: same results, and the caller's stream alone
    orders everything that follows (the results are read right after synchronising it)."""
    w = small_workload(SMALL[0])
    q, k, v = (x.cuda() for x in wl.make_qkv(w))
    do = wl.make_dout(w).cuda()
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, w.mask_mode, fuse_merge=True)
    one = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, w.mask_mode)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    for _ in range(3):
        two = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, w.mask_mode, aux_stream=side)
        torch.cuda.current_stream().synchronize()
        assert all(torch.equal(a, b) for a, b in zip(one, two))


def bwd_plan(tb, w, q, k, v, do, **kw):
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
    out, lse = tb.tasp_chunk_attn(qd, kd, vd, s, w.mask_mode, fuse_merge=True)
    return tb.ChunkAttnBwdPlan(s, qd, kd, vd, out, lse, dod, w.mask_mode, **kw)


def test_which_dkv_launches_are_split_by_query_head(tb):
    """A step's dk/dv launch with few, unequal key tiles runs one workgroup per key tile and query
    head and is followed by the launch that adds the partial sums up; seen from outside as one more
    launch per step among the profile's `other` launches (delta + clearing dq, and the cast of dq)."""
    w = small_workload(SMALL[0])                      # causal, 4 query heads per KV head
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    assert 2 < bwd_plan(tb, w, q, k, v, do).profile().other_launches <= 2 + w.n_ranks      # not where nobody sees a key
    assert bwd_plan(tb, w, q, k, v, do, fuse_steps=True).profile().other_launches == 3     # + the segment table
    w1 = small_workload(SMALL[5])                     # one query head per KV head: nothing to split by
    assert w1.Hq == w1.Hkv
    assert bwd_plan(tb, w1, *wl.make_qkv(w1), wl.make_dout(w1)).profile().other_launches == 2


def test_grouped_heads_step_by_step_with_equal_key_tiles(tb):
    """Without the mask every key tile costs the same, and 64 tiles x 8 KV heads fill the chip's 512
    workgroup slots (d = 64) exactly: this launch is NOT split, so the dk/dv kernel itself adds up the
    query heads of a group.  Every element, upstream gradient on sampled rows."""
    w = wl.Workload("bwd_full_n4_s32k_gqa2", 4, 1, 32768, 16, 8, 64, "bf16", wl.FULL, seed=wl.BASE_SEED + 733)
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    keep = wl.sample_rows(w, 16)
    sparse = torch.zeros_like(do)
    sparse[keep] = do[keep]
    plan = bwd_plan(tb, w, q, k, v, sparse)
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        assert plan.profile().other_launches == 2
    dq, dk, dv = plan.run()
    torch.cuda.synchronize()
    rq, rk, rv = oracle_grads(w, q, k, v, do, rows=keep)
    close("dq kept rows", dq[keep], rq)
    close("dk", dk, rk); close("dv", dv, rv)


def test_rows_without_upstream_gradient_get_none(tb):
    """dout = 0 on a row: its dq is exactly zero and it adds nothing to dk, dv (linearity in dout)."""
    w = small_workload(SMALL[0])
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    keep = [0, 5, 130, 255, 256, 300, w.L - 1]
    sparse = torch.zeros_like(do)
    sparse[keep] = do[keep]
    dq, dk, dv = forward_backward(tb, w, q, k, v, sparse)
    rq, rk, rv = oracle_grads(w, q, k, v, do, rows=keep)
    close("dq kept rows", dq[keep], rq)
    rest = np.setdiff1d(np.arange(w.L), keep)
    assert float(dq[rest].float().abs().max()) == 0.0
    close("dk", dk, rk); close("dv", dv, rv)


# ------------------------------------------------------------------ the benchmark's 128K workload, the launch configuration bench.py times
@pytest.mark.timeout(900)
@pytest.mark.parametrize("idx,n_random", [(1, 24), (2, 16), (3, 8)], ids=["128k_zigzag", "256k_full", "512k_zigzag_g8"])
def test_full_size_sparse_upstream_gradient(tb, capsys, idx, n_random):
    """Full size, every element of dq, dk and dv: the upstream gradient is non-zero on sampled rows
    only, which the oracle can afford (the kernels do the same work whatever dout holds).  The 128K
    workload is the configuration bench.py times; the 256K one has no mask (dk/dv launches never
    split), the 512K one eight query heads per KV head (dk/dv launches split by query head)."""
    w = wl.CONFIGS[idx]

    def say(msg):            # progress past pytest's capture: a silent minute reads as a hang on the GPU machine
        with capsys.disabled():
            print("[%s] %s" % (w.name, msg), flush=True)
    say("inputs")
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    keep = wl.sample_rows(w, n_random)
    sparse = torch.zeros_like(do)
    sparse[keep] = do[keep]
    say("oracle on %d rows" % len(keep))
    rq, rk, rv = oracle_grads(w, q, k, v, do, rows=keep, progress=say)
    rest = np.setdiff1d(np.arange(w.L), keep)
    for fuse_steps in (False, True):
        say("backward, fuse_steps=%s" % fuse_steps)
        dq, dk, dv = forward_backward(tb, w, q, k, v, sparse, fuse_steps=fuse_steps)
        close("dq kept rows", dq[keep], rq)
        assert float(dq[rest].float().abs().max()) == 0.0
        close("dk", dk, rk); close("dv", dv, rv)
        del dq, dk, dv
        torch.cuda.empty_cache()


def test_full_size_128k_dense_upstream_gradient(tb):
    """Full size, dense dout: dq on sampled rows one by one; for dk and dv the two sums that hold at
    any size (rows of p sum to one: sum_j dv_j = sum_i dout_i; rows of ds sum to zero: sum_j dk_j = 0)."""
    w = wl.CONFIGS[1]
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    dq, dk, dv = forward_backward(tb, w, q, k, v, do)
    rows = wl.sample_rows(w, 16)
    rq, _, _ = oracle_grads(w, q, k, v, do, rows=rows)
    close("dq sampled rows", dq[rows], rq)
    G = w.Hq // w.Hkv
    want = do.double().numpy().reshape(w.L, w.Hkv, G, w.d).sum(axis=(0, 2))          # [Hkv, d]
    got_v = dv.double().cpu().numpy().sum(axis=0)
    got_k = dk.double().cpu().numpy().sum(axis=0)
    # every dv_j, dk_j carries a bf16 rounding of relative 2^-9 with random sign
    slack_v = 6 * 2.0 ** -9 * float(np.sqrt((dv.double().cpu().numpy() ** 2).sum(axis=0)).max())
    slack_k = 6 * 2.0 ** -9 * float(np.sqrt((dk.double().cpu().numpy() ** 2).sum(axis=0)).max())
    assert np.abs(got_v - want).max() <= slack_v + 2.0 ** -8 * np.abs(want).max(), (np.abs(got_v - want).max(), slack_v)
    assert np.abs(got_k).max() <= slack_k + 1e-2, (np.abs(got_k).max(), slack_k)


# ------------------------------------------------------------------ fp32 inputs (the plain path): tight bar, no bf16 noise
FP32 = [
    ("cfg1", None),
    ("fp32_zz_n8", (8, 4, 8 * 2 * 40, 2, 2, 64, wl.ZIGZAG_CAUSAL)),
    ("fp32_full_d128_gqa", (4, 1, 4 * 70, 2, 1, 128, wl.FULL)),
    ("fp32_zz_n8_d128", (8, 7, 8 * 2 * 33, 4, 2, 128, wl.ZIGZAG_CAUSAL)),
]


@pytest.mark.parametrize("case", FP32, ids=[c[0] for c in FP32])
def test_fp32_all_outputs(tb, case):
    """fp32 in, fp32 out: forward then backward on the GPU against the exact gradient, every element,
    max-abs error at most 1e-4 of max(1, max|ref|) (the forward's bar for fp32)."""
    name, shape = case
    if shape is None:
        w = wl.CONFIGS[0]
    else:
        n, rank, S, Hq, Hkv, d, mode = shape
        w = wl.Workload("bwd_" + name, n, rank, S, Hq, Hkv, d, "fp32", mode, seed=wl.BASE_SEED + 950 + S % 89)
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    dq, dk, dv = forward_backward(tb, w, q, k, v, do)
    assert dq.dtype == torch.float32 and dk.dtype == torch.float32
    for nm, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), oracle_grads(w, q, k, v, do)):
        got = got.cpu().numpy().astype(np.float64)
        err = float(np.abs(got - ref).max())
        assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), (w.name, nm, err)


@pytest.mark.parametrize("fuse_steps", [False, True])
def test_backward_call_recorded_into_a_graph(tb, fuse_steps):
    """On one stream the backward call, too, enqueues kernels only: three graph replays with eager
    work between them against the eager result."""
    w = small_workload(SMALL[1])
    q, k, v = (x.cuda() for x in wl.make_qkv(w))
    do = wl.make_dout(w).cuda()
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, w.mask_mode, fuse_merge=True)
    plan = tb.ChunkAttnBwdPlan(s, q, k, v, out, lse, do, w.mask_mode, fuse_steps=fuse_steps)
    plan.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.run()
    for rep in range(3):
        do.copy_(torch.roll(do, shifts=rep + 1, dims=0))
        eager = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, w.mask_mode, fuse_steps=fuse_steps)
        torch.cuda.synchronize()
        for t in (plan.dq, plan.dk, plan.dv):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip((plan.dq, plan.dk, plan.dv), eager)), rep


def test_fp32_batched(tb):
    """The plain fp32 path with a batch of sequences: every element of every sequence at the fp32 bar."""
    B = 2
    ws = [wl.Workload("bwd_fp32_b%d" % b, 8, 1, 8 * 2 * 24, 2, 1, 64, "fp32", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 970 + b)
          for b in range(B)]
    data = [wl.make_qkv(w) + (wl.make_dout(w),) for w in ws]
    q, k, v, do = (torch.stack([x[i] for x in data]).cuda() for i in range(4))
    s = tb.tasp_schedule(8, 1)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, wl.ZIGZAG_CAUSAL)
    grads = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, wl.ZIGZAG_CAUSAL)
    torch.cuda.synchronize()
    for b in range(B):
        for nm, got, ref in zip(("dq", "dk", "dv"), grads, oracle_grads(ws[b], *data[b])):
            err = float(np.abs(got[b].cpu().numpy().astype(np.float64) - ref).max())
            assert err <= 1e-4 * max(1.0, float(np.abs(ref).max())), (b, nm, err)


# ------------------------------------------------------------------ the documented maxima
def test_thirty_two_ranks(tb):
    """N = 32, the most ranks one call takes (31 rings, 62 key segments per query block and step).
    The single-launch form is refused there: the later half-chunk of rank 17 meets
    31 x (17 + 2 x 14) = 1395 segments over all steps, more than TASP_MAX_FUSED_SEGMENTS."""
    w = wl.Workload("bwd_zz_n32", 32, 17, 64 * 36, 4, 2, 128, "bf16", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 761)
    q, k, v = wl.make_qkv(w)
    do = wl.make_dout(w)
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    out, lse = tb.tasp_chunk_attn(q.cuda(), k.cuda(), v.cuda(), s, w.mask_mode, fuse_merge=True)
    dq, dk, dv = tb.tasp_chunk_attn_bwd(q.cuda(), k.cuda(), v.cuda(), out, lse, do.cuda(), s, w.mask_mode)
    torch.cuda.synchronize()
    ro, rl = oracle_rows(w, q, k, v, range(w.L))
    assert np.abs(out.float().cpu().numpy() - ro).max() <= 2e-2 and np.abs(lse.cpu().numpy() - rl).max() <= 1e-3
    rq, rk, rv = oracle_grads(w, q, k, v, do, out=out.cpu())
    close("dq", dq, rq); close("dk", dk, rk); close("dv", dv, rv)
    for call in (lambda: tb.tasp_chunk_attn(q.cuda(), k.cuda(), v.cuda(), s, w.mask_mode, fuse_steps=True),
                 lambda: tb.tasp_chunk_attn_bwd(q.cuda(), k.cuda(), v.cuda(), out, lse, do.cuda(), s, w.mask_mode, fuse_steps=True)):
        with pytest.raises(tb.TaspError) as e:
            call()
        assert e.value.status == tb.EUNSUPPORTED_SHAPE


def test_kv_tensors_of_exactly_2_to_32_bytes(tb):
    """The largest K and V the bf16 kernels address (32-bit byte offsets): 2^21 tokens x 8 KV heads x
    128 x 2 bytes = 2^32 bytes each.  Rank 0 holds the first and the LAST half-chunk, so its later
    rows read every key up to the last byte.  Inputs are drawn on the GPU (seeded); the oracle gets the
    last head (the highest addresses) of sampled rows, the upstream gradient is non-zero on those rows."""
    S, H, d, n, rank = 1 << 21, 8, 128, 8, 0
    w1 = wl.Workload("max_kv_head7", n, rank, S, 1, 1, d, "bf16", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 787)
    L = S // n
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w1.seed)
    def draw(rows):
        t = torch.empty((rows, H, d), dtype=torch.bfloat16, device="cuda")
        for a in range(0, rows, 1 << 18):
            b = min(rows, a + (1 << 18))
            t[a:b] = torch.randn((b - a, H, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        return t
    q, k, v = draw(L), draw(S), draw(S)
    assert k.numel() * k.element_size() == 1 << 32
    keep = wl.sample_rows(w1, 8)
    assert L - 1 in keep
    do = torch.zeros_like(q)
    do[keep] = torch.randn((len(keep), H, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    s = tb.tasp_schedule(n, rank)
    h = H - 1
    q1, k1, v1, do1 = (t[:, h:h + 1].cpu() for t in (q, k, v, do))
    ro, rl = oracle_rows(w1, q1, k1, v1, keep)
    rq = rk = rv = None
    for fuse_steps in (False, True):
        out, lse = tb.tasp_chunk_attn(q, k, v, s, wl.ZIGZAG_CAUSAL, fuse_merge=True, fuse_steps=fuse_steps)
        torch.cuda.synchronize()
        eo = np.abs(out[keep, h:h + 1].float().cpu().numpy() - ro).max()
        el = np.abs(lse[keep, h:h + 1].cpu().numpy() - rl).max()
        assert eo <= 2e-2 and el <= 1e-3, (fuse_steps, eo, el)
        dq, dk, dv = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, wl.ZIGZAG_CAUSAL, fuse_steps=fuse_steps)
        torch.cuda.synchronize()
        if rq is None:
            rq, rk, rv = oracle_grads(w1, q1, k1, v1, do1, rows=keep, out=out[:, h:h + 1].cpu())
        close("dq kept rows", dq[keep, h:h + 1], rq)
        close("dk last head", dk[:, h:h + 1], rk); close("dv last head", dv[:, h:h + 1], rv)
        del out, lse, dq, dk, dv


def test_sequence_just_below_2_to_24_tokens(tb):
    """The longest sequence the bf16 kernels take (token index times row bytes by a 24-bit multiply):
    S = 2^24 - 64 tokens, one head of 64 columns, 32 ranks; rank 0 reads up to the last token.  Forward
    and backward step by step (the single-launch form is refused at this rank count), sampled rows."""
    S, d, n, rank = (1 << 24) - 64, 64, 32, 0
    w1 = wl.Workload("max_tokens", n, rank, S, 1, 1, d, "bf16", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 797)
    L, Hh = S // n, S // (2 * n)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w1.seed)
    def draw(rows):
        t = torch.empty((rows, 1, d), dtype=torch.bfloat16, device="cuda")
        for a in range(0, rows, 1 << 21):
            b = min(rows, a + (1 << 21))
            t[a:b] = torch.randn((b - a, 1, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        return t
    q, k, v = draw(L), draw(S), draw(S)
    keep = sorted({0, Hh - 1, Hh, L - 1} | {int(x) for x in torch.randint(0, L, (2,), generator=torch.Generator().manual_seed(5))})
    do = torch.zeros_like(q)
    do[keep] = torch.randn((len(keep), 1, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    s = tb.tasp_schedule(n, rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, wl.ZIGZAG_CAUSAL, fuse_merge=True)
    dq, dk, dv = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, wl.ZIGZAG_CAUSAL)
    torch.cuda.synchronize()
    qc, kc, vc, doc = q.cpu(), k.cpu(), v.cpu(), do.cpu()
    ro, rl = oracle_rows(w1, qc, kc, vc, keep)
    eo = np.abs(out[keep].float().cpu().numpy() - ro).max()
    el = np.abs(lse[keep].cpu().numpy() - rl).max()
    assert eo <= 2e-2 and el <= 1e-3, (eo, el)
    rq, rk, rv = oracle_grads(w1, qc, kc, vc, doc, rows=keep, out=out.cpu())
    close("dq kept rows", dq[keep], rq)
    close("dk", dk, rk); close("dv", dv, rv)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_largest_batch(tb, dtype):
    """65535 sequences in one call, the most it takes; tiny ones (N = 4, 8 tokens, two rows a rank).
    The first, a middle and the last sequence against the oracle, forward and backward."""
    B, n, rank, S, Hq, Hkv, d = 65535, 4, 2, 8, 2, 1, 64
    w = wl.Workload("max_batch_" + dtype, n, rank, S, Hq, Hkv, d, dtype, wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 811)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    draw = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(w.torch_dtype)
    q, k, v, do = draw(B, w.L, Hq, d), draw(B, S, Hkv, d), draw(B, S, Hkv, d), draw(B, w.L, Hq, d)
    s = tb.tasp_schedule(n, rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, w.mask_mode, fuse_merge=True)
    dq, dk, dv = tb.tasp_chunk_attn_bwd(q, k, v, out, lse, do, s, w.mask_mode)
    torch.cuda.synchronize()
    tol_o, tol_l = (2e-2, 1e-3) if dtype == "bf16" else (1e-4, 1e-4)
    for b in (0, 31000, B - 1):
        qb, kb, vb, dob = q[b].cpu(), k[b].cpu(), v[b].cpu(), do[b].cpu()
        ro, rl = oracle_rows(w, qb, kb, vb, range(w.L))
        assert np.abs(out[b].float().cpu().numpy() - ro).max() <= tol_o and np.abs(lse[b].cpu().numpy() - rl).max() <= tol_l
        rq, rk, rv = oracle_grads(w, qb, kb, vb, dob, out=out[b].cpu())
        if dtype == "bf16":
            close("dq", dq[b], rq); close("dk", dk[b], rk); close("dv", dv[b], rv)
        else:
            for got, ref in ((dq[b], rq), (dk[b], rk), (dv[b], rv)):
                assert np.abs(got.cpu().numpy() - ref).max() <= 1e-4 * max(1.0, np.abs(ref).max())
