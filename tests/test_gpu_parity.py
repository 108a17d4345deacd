"""Parity of the HIP path (through the C ABI) with the fp64 oracle on the same seeded inputs.

Tolerances (max-abs): fp32 inputs 1e-4 on out and lse; bf16 inputs 2e-2 on out, 1e-3 on lse."""
import numpy as np
import pytest
import torch

from oracle import attention as att
from oracle import schedule as sch
from paper_2509_26541_amd import workloads as wl
from tests.helpers import max_abs, oracle_rows

pytestmark = pytest.mark.gpu

TOL = {"fp32": (1e-4, 1e-4), "bf16": (2e-2, 1e-3)}


@pytest.fixture(scope="module")
def tb():
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2509_26541_amd import binding
    return binding


def run_gpu(tb, w, q, k, v, **kw):
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    out, lse = tb.tasp_chunk_attn(q.cuda(), k.cuda(), v.cuda(), s, w.mask_mode, **kw)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), lse.cpu().numpy()


def check(w, out, lse, ref_o, ref_l, rows, heads=None):
    heads = list(range(w.Hq)) if heads is None else heads
    tol_o, tol_l = TOL[w.dtype]
    eo = max_abs(out[np.ix_(rows, heads)], ref_o)
    el = max_abs(lse[np.ix_(rows, heads)], ref_l)
    assert np.all(np.isfinite(lse[np.ix_(rows, heads)]))
    assert eo <= tol_o and el <= tol_l, "%s: out err %.3e (tol %g), lse err %.3e (tol %g)" % (w.name, eo, tol_o, el, tol_l)
    return eo, el


# ------------------------------------------------------------------ config 1: every row, fp32
@pytest.mark.parametrize("fuse", [False, True])
def test_cfg1_fp32_all_rows(tb, fuse):
    w = wl.CONFIGS[0]
    q, k, v = wl.make_qkv(w)
    out, lse = run_gpu(tb, w, q, k, v, fuse_merge=fuse)
    rows = list(range(w.L))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    check(w, out, lse, ref_o, ref_l, rows)


# ------------------------------------------------------------------ small cases, every row
SMALL = [
    # name, base config index, N, rank, S, Hq, Hkv, d
    ("bf16_zz_n8", 1, 8, 3, 4096, 8, 2, 128),
    ("bf16_zz_n8_ragged", 1, 8, 6, 8 * 2 * 200, 4, 2, 128),     # H = 200: ragged query and key tiles
    ("bf16_zz_n8_tiny", 1, 8, 0, 112, 2, 1, 128),               # sub-chunks of 1 token
    ("bf16_zz_n8_one_row", 1, 8, 5, 16, 2, 2, 128),             # the smallest sequence: one row per half-chunk, most sub-chunks empty
    ("bf16_full_n4_one_row", 2, 4, 3, 4, 2, 1, 64),             # L = 1
    ("bf16_full_n8", 2, 8, 0, 8 * 331, 4, 4, 128),              # L = 331, pieces of 47/48
    ("bf16_full_n4", 2, 4, 2, 4 * 512, 4, 1, 128),
    ("bf16_zz_n16", 3, 16, 5, 16 * 2 * 96, 8, 1, 128),
    ("bf16_zz_n8_outliers", 4, 8, 7, 4096, 4, 2, 128),
    ("bf16_zz_d64", 1, 8, 2, 4096, 4, 2, 64),
    ("bf16_full_d64", 2, 8, 5, 8 * 200, 2, 2, 64),
    ("bf16_zz_d64_w12", 1, 8, 2, 16 * 768, 2, 1, 64),           # half-chunks of 768 rows: the twelve-wavefront variant (384-row tiles)
    ("bf16_full_d64_w12", 2, 8, 6, 8 * 1152, 2, 2, 64),         # L = 1152 = 3 x 384
    ("bf16_zz_d64_mha12", 1, 8, 1, 2048, 12, 12, 64),          # 12 KV heads: pairs of XCDs share three heads
    ("bf16_full_gqa_kv6", 2, 8, 4, 8 * 256, 12, 6, 128),       # 6 KV heads: four XCDs share three heads
    ("bf16_zz_kv3", 1, 8, 6, 8 * 2 * 72, 3, 3, 128),           # 3 KV heads: all XCDs share them
    ("fp32_zz_n8", 0, 8, 4, 8 * 2 * 40, 2, 2, 64),
    ("fp32_full_d128", 0, 4, 1, 4 * 70, 2, 1, 128),
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
@pytest.mark.parametrize("fuse", [False, True])
def test_small_all_rows(tb, case, fuse):
    name, base, n, rank, S, Hq, Hkv, d = case
    b = wl.CONFIGS[base]
    w = wl.Workload(name, n, rank, S, Hq, Hkv, d, "fp32" if name.startswith("fp32") else "bf16",
                    wl.ZIGZAG_CAUSAL if "_zz_" in name else wl.FULL, k_scale=b.k_scale,
                    outlier_frac=0.05 if "outliers" in name else 0.0, seed=b.seed + 100)
    q, k, v = wl.make_qkv(w)
    out, lse = run_gpu(tb, w, q, k, v, fuse_merge=fuse)
    rows = list(range(w.L))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    check(w, out, lse, ref_o, ref_l, rows)


SMALL_BF16 = [c for c in SMALL if not c[0].startswith("fp32")]


@pytest.mark.parametrize("case", SMALL_BF16, ids=[c[0] for c in SMALL_BF16])
def test_small_all_rows_single_launch(tb, case):
    """fuse_steps: one launch walks the sub-chunks of all steps in arrival order."""
    name, base, n, rank, S, Hq, Hkv, d = case
    b = wl.CONFIGS[base]
    w = wl.Workload(name, n, rank, S, Hq, Hkv, d, "bf16", wl.ZIGZAG_CAUSAL if "_zz_" in name else wl.FULL,
                    k_scale=b.k_scale, outlier_frac=0.05 if "outliers" in name else 0.0, seed=b.seed + 100)
    q, k, v = wl.make_qkv(w)
    rows = list(range(w.L))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    for kw in ({}, {"order": tb.ORDER_RING}):
        out, lse = run_gpu(tb, w, q, k, v, fuse_steps=True, **kw)
        check(w, out, lse, ref_o, ref_l, rows)


SMALL_FP32 = [c for c in SMALL if c[0].startswith("fp32")]


@pytest.mark.parametrize("case", [("cfg1",)] + SMALL_FP32, ids=["cfg1"] + [c[0] for c in SMALL_FP32])
def test_fp32_single_launch_all_rows(tb, case):
    """fuse_steps with fp32 inputs: workload 1 (four launches become one) and the small fp32 cases."""
    if case[0] == "cfg1":
        w = wl.CONFIGS[0]
    else:
        name, base, n, rank, S, Hq, Hkv, d = case
        w = wl.Workload(name, n, rank, S, Hq, Hkv, d, "fp32", wl.ZIGZAG_CAUSAL if "_zz_" in name else wl.FULL,
                        seed=wl.CONFIGS[base].seed + 100)
    q, k, v = wl.make_qkv(w)
    rows = list(range(w.L))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    for kw in ({}, {"order": tb.ORDER_RING}):
        out, lse = run_gpu(tb, w, q, k, v, fuse_steps=True, **kw)
        check(w, out, lse, ref_o, ref_l, rows)


def test_backward_single_launch_refuses_fp32(tb):
    w = wl.CONFIGS[0]                                    # fp32: the plain backward path walks step by step
    q, k, v = (x.cuda() for x in wl.make_qkv(w))
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, w.mask_mode)
    with pytest.raises(tb.TaspError) as e:
        tb.tasp_chunk_attn_bwd(q, k, v, out, lse, torch.ones_like(q), s, w.mask_mode, fuse_steps=True)
    assert e.value.status == tb.EUNSUPPORTED_SHAPE


def test_ring_order_gives_the_same_result(tb):
    w = wl.Workload("ring", 8, 3, 4096, 8, 2, 128, "bf16", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 77)
    q, k, v = wl.make_qkv(w)
    out, lse = run_gpu(tb, w, q, k, v, order=tb.ORDER_RING)
    rows = list(range(w.L))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    check(w, out, lse, ref_o, ref_l, rows)


# ------------------------------------------------------------------ one step at a time
@pytest.mark.parametrize("mode", [wl.FULL, wl.ZIGZAG_CAUSAL])
def test_step_partials_match_algorithm_3(tb, mode):
    """tasp_step_attn against the oracle's per-step partial (out_s, lse_s), including rows that see
    nothing at a step (lse = -inf, out = 0)."""
    # rank 0: every remote sub-chunk comes from a higher rank, so the first half-chunk's rows see
    # nothing after step 0 in the zig-zag layout
    w = wl.Workload("steps", 8, 0, 8 * 2 * 72, 4, 2, 128, "bf16", mode, seed=wl.BASE_SEED + 55)
    q, k, v = wl.make_qkv(w)
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    pos = sch.local_positions(w.n_ranks, w.rank, w.S, mode)
    rows = list(range(0, w.L, 5))
    h = 3
    g = h * w.Hkv // w.Hq
    _, _, partials = att.stepwise_rows(q[rows, h].double().numpy(), [pos[r] for r in rows], k[:, g].double().numpy(),
                                       v[:, g].double().numpy(), w.n_ranks, w.rank, mode)
    saw_empty = False
    for step in range(w.n_ranks):
        o, l = tb.tasp_step_attn(qd, kd, vd, s, mode, step)
        torch.cuda.synchronize()
        o, l = o.cpu().numpy()[rows, h], l.cpu().numpy()[rows, h]
        ref_o, ref_l = partials[step]
        assert np.array_equal(np.isneginf(l), np.isneginf(ref_l))
        saw_empty |= bool(np.any(np.isneginf(ref_l)))
        assert max_abs(l, ref_l) <= 1e-3 and max_abs(o, ref_o) <= 2e-2
        assert np.all(o[np.isneginf(l)] == 0)
    assert saw_empty == (mode == wl.ZIGZAG_CAUSAL)


# ------------------------------------------------------------------ update_out_lse kernel
def test_lse_merge_kernel(tb):
    rng = np.random.default_rng(11)
    rows, heads, d = 777, 5, 128
    oa, ob = rng.standard_normal((rows, heads, d)), rng.standard_normal((rows, heads, d))
    la, lb = rng.standard_normal((rows, heads)) * 6, rng.standard_normal((rows, heads)) * 6
    la[::7] = -np.inf
    lb[::5] = -np.inf                      # every 35th row: both empty
    oa[np.isneginf(la)] = 0
    ob[np.isneginf(lb)] = 0
    la[3, 1], lb[3, 1] = 50.0, -60.0       # huge gap
    t = [torch.tensor(x, dtype=torch.float32).cuda() for x in (oa, la, ob, lb)]
    ref_o, ref_l = att.lse_merge(t[0].cpu().double().numpy(), t[1].cpu().double().numpy(),
                                 t[2].cpu().double().numpy(), t[3].cpu().double().numpy())
    tb.tasp_lse_merge(*t)
    torch.cuda.synchronize()
    got_o, got_l = t[0].cpu().numpy(), t[1].cpu().numpy()
    assert np.array_equal(np.isneginf(got_l), np.isneginf(ref_l))
    assert max_abs(got_l, ref_l) <= 1e-5 and max_abs(got_o, ref_o) <= 1e-5
    assert np.all(got_o[np.isneginf(got_l)] == 0)
    # d = 64 and a ragged count
    t = [torch.tensor(x[:33, :3, :64] if x.ndim == 3 else x[:33, :3], dtype=torch.float32).contiguous().cuda()
         for x in (oa, la, ob, lb)]
    ref_o, ref_l = att.lse_merge(*[x.cpu().double().numpy() for x in (t[0], t[1], t[2], t[3])])
    tb.tasp_lse_merge(*t)
    torch.cuda.synchronize()
    assert max_abs(t[1].cpu().numpy(), ref_l) <= 1e-5 and max_abs(t[0].cpu().numpy(), ref_o) <= 1e-5


def test_lse_merge_many_kernel(tb):
    """One pass over N partials against the oracle's closed form; also in place on the first partial
    and against the fold of the pairwise kernel."""
    rng = np.random.default_rng(12)
    for rows, heads, d, n in [(301, 5, 128, 8), (33, 3, 64, 3), (7, 2, 128, 1), (64, 4, 128, 16)]:
        os_ = [rng.standard_normal((rows, heads, d)) for _ in range(n)]
        ls = [rng.standard_normal((rows, heads)) * 6 for _ in range(n)]
        for i in range(n):
            ls[i][i::(n + 2)] = -np.inf                # empty partials here and there
            os_[i][np.isneginf(ls[i])] = 0
        for l in ls:
            l[5 % rows] = -np.inf                      # a row no partial has seen
        for o in os_:
            o[5 % rows] = 0
        ls[0][2 % rows, 0] = 70.0                      # one partial dominates
        to = [torch.tensor(x, dtype=torch.float32).cuda() for x in os_]
        tl = [torch.tensor(x, dtype=torch.float32).cuda() for x in ls]
        ref_o, ref_l = att.lse_merge_many([x.cpu().double().numpy() for x in to], [x.cpu().double().numpy() for x in tl])
        got_o, got_l = tb.tasp_lse_merge_many(to, tl)
        torch.cuda.synchronize()
        go, gl = got_o.cpu().numpy(), got_l.cpu().numpy()
        assert np.array_equal(np.isneginf(gl), np.isneginf(ref_l))
        assert np.isneginf(gl[5 % rows]).all() and np.all(go[5 % rows] == 0)
        assert max_abs(gl, ref_l) <= 1e-5 and max_abs(go, ref_o) <= 1e-5
        # the fold of the pairwise kernel gives the same up to rounding
        fo, fl = to[0].clone(), tl[0].clone()
        for i in range(1, n):
            tb.tasp_lse_merge(fo, fl, to[i], tl[i])
        torch.cuda.synchronize()
        assert max_abs(fl.cpu().numpy(), gl) <= 2e-5 and max_abs(fo.cpu().numpy(), go) <= 2e-5
        # in place on the first partial
        tb.tasp_lse_merge_many(to, tl, o_out=to[0], lse_out=tl[0])
        torch.cuda.synchronize()
        assert np.array_equal(to[0].cpu().numpy(), go) and np.array_equal(tl[0].cpu().numpy(), gl)


def test_calibration_mfma_runs(tb):
    flops = tb.tasp_calibration_mfma(10)
    torch.cuda.synchronize()
    assert flops == 2048 * 8 * 10 * 32 * 32768.0


# ------------------------------------------------------------------ full-size configs, sampled rows
# ------------------------------------------------------------------ a batch of sequences in one call
BATCHED = [
    ("bf16_zz_b3", 8, 3, 8 * 2 * 100, 4, 2, 128, "bf16", wl.ZIGZAG_CAUSAL, 3),
    ("bf16_full_b2_d64", 8, 6, 8 * 150, 2, 2, 64, "bf16", wl.FULL, 2),
    ("fp32_zz_b4", 4, 1, 4 * 2 * 30, 2, 1, 64, "fp32", wl.ZIGZAG_CAUSAL, 4),
]


def test_calibration_issue_prices_the_vector_port(tb):
    """The figures bench.py uses for the vector issue port (matrix 12, vector 4, exponential 8, KiB of
    LDS data 4 cycles) against what the calibration kernel measures on this GPU."""
    import bench
    got = bench.measure_port_cycles(tb)
    for name, want in (("mfma", 12.0), ("valu", 4.0), ("exp", 8.0), ("lds_kib", 4.0)):
        assert abs(got[name] - want) <= 0.25 * want, got
    with pytest.raises(tb.TaspError):
        tb.tasp_calibration_issue(0, 5)


def test_paper_grid_shape_batched(tb):
    """A shape of the paper's own grid (Sec. 5.1.2: 12 heads of 64, its shortest sequence 3K) with a
    batch of 3: every row of every sequence against the oracle."""
    ws = [wl.paper_grid(12, 3072, seed_offset=1000 * b) for b in range(3)]
    qkv = [wl.make_qkv(w) for w in ws]
    q, k, v = (torch.stack([x[i] for x in qkv]).cuda() for i in range(3))
    s = tb.tasp_schedule(ws[0].n_ranks, ws[0].rank)
    for fuse in (False, True):
        out, lse = tb.tasp_chunk_attn(q, k, v, s, ws[0].mask_mode, fuse_merge=fuse)
        torch.cuda.synchronize()
        rows = list(range(ws[0].L))
        for b in range(3):
            ref_o, ref_l = oracle_rows(ws[b], *qkv[b], rows)
            check(ws[b], out[b].float().cpu().numpy(), lse[b].cpu().numpy(), ref_o, ref_l, rows)


def test_single_launch_with_persistent_workgroups(tb):
    """d = 64 and all steps in one launch with more work items (2 tasks x 12 heads x 16 sequences = 384)
    than CUs: one persistent workgroup per CU takes its items in turn (two rounds, the second
    incomplete).  Every row of three of the sequences against the oracle, the others against the
    step-by-step call."""
    B = 16
    ws = [wl.paper_grid(12, 3072, seed_offset=1000 * b) for b in range(B)]
    qkv = [wl.make_qkv(w) for w in ws]
    q, k, v = (torch.stack([x[i] for x in qkv]).cuda() for i in range(3))
    s = tb.tasp_schedule(ws[0].n_ranks, ws[0].rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, ws[0].mask_mode, fuse_steps=True)
    ref_out, ref_lse = tb.tasp_chunk_attn(q, k, v, s, ws[0].mask_mode, fuse_merge=True)
    torch.cuda.synchronize()
    rows = list(range(ws[0].L))
    for b in (0, 7, 15):
        ref_o, ref_l = oracle_rows(ws[b], *qkv[b], rows)
        check(ws[b], out[b].float().cpu().numpy(), lse[b].cpu().numpy(), ref_o, ref_l, rows)
    assert float((lse - ref_lse).abs().max()) <= 1e-4 and float((out.float() - ref_out.float()).abs().max()) <= 2e-2


@pytest.mark.parametrize("case", BATCHED, ids=[c[0] for c in BATCHED])
@pytest.mark.parametrize("fuse", [False, True])
def test_batched_call(tb, case, fuse):
    """B sequences in one call (the paper's shape grid has a batch dimension): every sequence against
    the oracle, and bit-identical to B separate calls."""
    name, n, rank, S, Hq, Hkv, d, dtype, mode, B = case
    ws = [wl.Workload("%s_%d" % (name, b), n, rank, S, Hq, Hkv, d, dtype, mode, seed=wl.BASE_SEED + 500 + 7 * b)
          for b in range(B)]
    qkv = [wl.make_qkv(w) for w in ws]
    q = torch.stack([x[0] for x in qkv]).cuda()
    k = torch.stack([x[1] for x in qkv]).cuda()
    v = torch.stack([x[2] for x in qkv]).cuda()
    s = tb.tasp_schedule(n, rank)
    out, lse = tb.tasp_chunk_attn(q, k, v, s, mode, fuse_merge=fuse)
    torch.cuda.synchronize()
    assert tuple(out.shape) == tuple(q.shape) and tuple(lse.shape) == tuple(q.shape[:-1])
    if dtype == "bf16":                      # all steps in one launch, batched: same bar (checked below via out1/lse1)
        out1, lse1 = tb.tasp_chunk_attn(q, k, v, s, mode, fuse_steps=True)
        torch.cuda.synchronize()
        assert float((out1.float() - out.float()).abs().max()) <= 2e-2 and float((lse1 - lse).abs().max()) <= 1e-3
    rows = list(range(ws[0].L))
    for b in range(B):
        ref_o, ref_l = oracle_rows(ws[b], *qkv[b], rows)
        check(ws[b], out[b].float().cpu().numpy(), lse[b].cpu().numpy(), ref_o, ref_l, rows)
        o1, l1 = tb.tasp_chunk_attn(q[b].contiguous(), k[b].contiguous(), v[b].contiguous(), s, mode, fuse_merge=fuse)
        torch.cuda.synchronize()
        assert torch.equal(o1, out[b]) and torch.equal(l1, lse[b])
    # the partial of one step, batched
    o_s, l_s = tb.tasp_step_attn(q, k, v, s, mode, 2)
    o_1, l_1 = tb.tasp_step_attn(q[B - 1].contiguous(), k[B - 1].contiguous(), v[B - 1].contiguous(), s, mode, 2)
    torch.cuda.synchronize()
    assert torch.equal(o_s[B - 1], o_1) and torch.equal(l_s[B - 1], l_1)


# ------------------------------------------------------------------ (m-K_m-m)^u schedules (Sec. 3.1.3)
MULTINODE = [
    # name, ranks per node, nodes, rank, S, Hq, Hkv, d, mask
    ("mn_4x2_zz", 4, 2, 5, 8 * 2 * 200, 4, 2, 128, wl.ZIGZAG_CAUSAL),      # 4 sub-chunks of 50 tokens
    ("mn_8x2_zz", 8, 2, 9, 16 * 2 * 100, 4, 1, 128, wl.ZIGZAG_CAUSAL),     # pieces of 12/13 tokens
    ("mn_8x2_full", 8, 2, 0, 16 * 150, 2, 2, 128, wl.FULL),
    ("mn_2x3_zz_d64", 2, 3, 4, 6 * 2 * 96, 2, 2, 64, wl.ZIGZAG_CAUSAL),
]


@pytest.mark.parametrize("case", MULTINODE, ids=[c[0] for c in MULTINODE])
@pytest.mark.parametrize("fuse", [False, True])
def test_small_multinode_schedule_all_rows(tb, case, fuse):
    """The result does not depend on the ring table; with m rings a step concatenates m sub-chunks."""
    name, m, u, rank, S, Hq, Hkv, d, mode = case
    w = wl.Workload(name, m * u, rank, S, Hq, Hkv, d, "bf16", mode, seed=wl.BASE_SEED + 300 + m + u)
    q, k, v = wl.make_qkv(w)
    s = tb.tasp_schedule_multinode(m, u, rank)
    assert s.n_rings == m
    rows = list(range(w.L))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    for fuse_steps in (False, True):
        out, lse = tb.tasp_chunk_attn(q.cuda(), k.cuda(), v.cuda(), s, mode, fuse_merge=fuse, fuse_steps=fuse_steps)
        torch.cuda.synchronize()
        check(w, out.float().cpu().numpy(), lse.cpu().numpy(), ref_o, ref_l, rows)
    # the partial of one step against the oracle's partial over that step's tokens
    rings = sch.multinode_rings(m, u)
    step = 1 + (rank % (m * u - 1))
    o_s, l_s = tb.tasp_step_attn(q.cuda(), k.cuda(), v.cuda(), s, mode, step)
    torch.cuda.synchronize()
    toks = att.step_tokens(m * u, rank, S, mode, rings, step)
    pos = sch.local_positions(m * u, rank, S, mode)
    kk, vv = k[:, 0].double().numpy(), v[:, 0].double().numpy()
    for r in (0, w.L // 2 - 1, w.L // 2, w.L - 1):
        ro, rl = att.partial_over_tokens(q[r, 0].double().numpy(), pos[r], kk, vv, toks, mode == wl.ZIGZAG_CAUSAL,
                                         1.0 / np.sqrt(d))
        assert max_abs(l_s[r, 0].cpu().numpy(), rl) <= 1e-3
        assert max_abs(o_s[r, 0].cpu().numpy(), ro) <= 2e-2


@pytest.mark.timeout(900)
def test_full_size_multinode_8x2_sampled_rows(tb):
    """Workload 4's shape (16 ranks as 2 nodes of 8) with the (8-K_8-8)^2 schedule: 8 sub-chunks per
    step instead of 15."""
    w = wl.CONFIGS[3]
    say = lambda msg: print("[%s, (8-K_8-8)^2] %s" % (w.name, msg), flush=True)
    say("generating inputs")
    q, k, v = wl.make_qkv(w)
    s = tb.tasp_schedule_multinode(8, 2, w.rank)
    say("running tasp_chunk_attn")
    out, lse = tb.tasp_chunk_attn(q.cuda(), k.cuda(), v.cuda(), s, w.mask_mode, fuse_merge=True)
    torch.cuda.synchronize()
    out, lse = out.float().cpu().numpy(), lse.cpu().numpy()
    torch.cuda.empty_cache()
    rows = wl.sample_rows(w, 8)[:16]
    say("oracle: %d rows x all heads" % len(rows))
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    check(w, out, lse, ref_o, ref_l, rows)
    assert np.all(np.isfinite(lse)) and np.all(np.isfinite(out))


# (workload index, random rows checked on every head, random rows checked on one head per KV group);
# on top of these come the tile-edge rows of sample_rows and the rows next to sub-chunk bounds
FULL_SIZE = [(1, 64, 1024), (2, 64, 1024), (3, 32, 512), (4, 48, 768)]


def subchunk_edge_rows(w):
    """Local rows whose own position sits at a bound of a sub-chunk of the rank's own chunk (the last
    row of a piece and the first of the next, eq. (3), (5), (6)): there the causal diagonal and a
    segment bound of step 0 coincide."""
    pos = np.asarray(sch.local_positions(w.n_ranks, w.rank, w.S, w.mask_mode), dtype=np.int64)
    local_of = {int(p): i for i, p in enumerate(pos)}
    rows = set()
    for ring in range(w.n_ranks - 1):
        for a, b in sch.subchunk_ranges(w.n_ranks, w.S, w.mask_mode, ring, w.rank):
            for p in (a - 1, a, b - 1, b):
                if p in local_of:
                    rows.add(local_of[p])
    return sorted(rows)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("idx,n_all_heads,n_one_head", FULL_SIZE, ids=[wl.CONFIGS[i[0]].name for i in FULL_SIZE])
def test_full_size_sampled_rows(tb, capsys, idx, n_all_heads, n_one_head):
    """The launch configuration the benchmark times, checked on sampled rows the oracle computes one
    by one: tile-edge and half-chunk-edge rows plus seeded random rows on every head; those, the rows
    at the bounds of the rank's own sub-chunks and a larger random set on one head per KV group.
    Random rows: 64 + 1024 for the 128K and 256K workloads, 32 + 512 at 512K (64 query heads),
    48 + 768 at 1M (the oracle is dense fp64 over all keys of every sampled row)."""
    w = wl.CONFIGS[idx]
    def say(msg):            # progress past pytest's capture: a silent minute reads as a hang on the GPU machine
        with capsys.disabled():
            print("[%s] %s" % (w.name, msg), flush=True)
    say("generating inputs")
    q, k, v = wl.make_qkv(w)
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    say("running tasp_chunk_attn (merge kernel, fused merge, all steps in one launch)")
    results = {}
    for fuse in (False, True, "one launch"):
        out, lse = tb.tasp_chunk_attn(qd, kd, vd, s, w.mask_mode, fuse_merge=bool(fuse), fuse_steps=fuse == "one launch")
        torch.cuda.synchronize()
        results[fuse] = (out.float().cpu().numpy(), lse.cpu().numpy())
    del qd, kd, vd
    torch.cuda.empty_cache()
    rows_a = wl.sample_rows(w, n_all_heads)                     # tile-edge rows + n_all_heads random ones
    edge = subchunk_edge_rows(w)
    rows_b = sorted(set(wl.sample_rows(w, n_one_head, seed_offset=1)) | set(edge))
    G = w.Hq // w.Hkv
    heads_b = [g * G + (g % G) for g in range(w.Hkv)]
    say("oracle: %d rows x all heads" % len(rows_a))
    ref_a = oracle_rows(w, q, k, v, rows_a)
    say("oracle: %d rows x %d heads" % (len(rows_b), len(heads_b)))
    parts = []
    for c0 in range(0, len(rows_b), 256):       # in pieces, with a progress line each
        parts.append(oracle_rows(w, q, k, v, rows_b[c0:c0 + 256], heads_b))
        say("  ... %d rows done" % min(len(rows_b), c0 + 256))
    ref_b = (np.concatenate([x[0] for x in parts]), np.concatenate([x[1] for x in parts]))
    say("comparing")
    for fuse, (out, lse) in results.items():
        check(w, out, lse, ref_a[0], ref_a[1], rows_a)
        check(w, out, lse, ref_b[0], ref_b[1], rows_b, heads_b)
    # properties that hold at any size: finite everywhere, the two merge paths agree closely
    for out, lse in results.values():
        assert np.all(np.isfinite(lse)) and np.all(np.isfinite(out))
    assert max_abs(results[False][1], results[True][1]) <= 1e-4
    assert max_abs(results["one launch"][1], results[True][1]) <= 1e-4


@pytest.mark.timeout(600)
def test_long_row_with_one_dominant_early_key(tb):
    """Half a million keys, the very first of which outweighs each of the others by e^20 while all
    the others together still make up 1e-3 of the sum: a single fp32 accumulator would swallow every
    one of them (each is below half an ulp of it) and lose 1e-3 in lse.  The bar here is 1e-4."""
    n, rank, S, d = 8, 0, 8 * 65536, 64
    w = wl.Workload("dominant_first_key", n, rank, S, 1, 1, d, "bf16", wl.FULL, seed=wl.BASE_SEED + 4242)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(w.seed)
    u = torch.full((d,), 1.0 / 8.0)                                   # unit vector
    q = (torch.randn((w.L, 1, d), generator=gen) + 4.0 * u).to(torch.bfloat16)
    k = (0.3 * torch.randn((S, 1, d), generator=gen)).to(torch.bfloat16)
    v = torch.randn((S, 1, d), generator=gen).to(torch.bfloat16)
    k[0, 0] = (40.0 * u).to(torch.bfloat16)                           # score 40 * 4 / sqrt(64) = 20 above the rest
    rows = wl.sample_rows(w, 12)[:20]
    ref_o, ref_l = oracle_rows(w, q, k, v, rows)
    s = tb.tasp_schedule(n, rank)
    for kw in (dict(fuse_merge=True), dict(fuse_steps=True)):
        out, lse = tb.tasp_chunk_attn(q.cuda(), k.cuda(), v.cuda(), s, w.mask_mode, **kw)
        torch.cuda.synchronize()
        err = max_abs(lse.cpu().numpy()[rows], ref_l)
        assert err <= 1e-4, (kw, err)
        assert max_abs(out.float().cpu().numpy()[rows], ref_o) <= 2e-2


@pytest.mark.parametrize("mode", ["merge_kernel", "fused_merge", "single_launch"])
def test_forward_call_recorded_into_a_graph(tb, mode):
    """The forward call enqueues kernels only (no memset, no copy from host memory), so it can be
    recorded into a HIP graph: three replays, with eager work and synchronisation between them and
    fresh inputs each time, against the eager result."""
    w = wl.Workload("graph", 8, 5, 8 * 2 * 160, 4, 2, 128, "bf16", wl.ZIGZAG_CAUSAL, seed=wl.BASE_SEED + 31)
    q, k, v = (x.cuda() for x in wl.make_qkv(w))
    s = tb.tasp_schedule(w.n_ranks, w.rank)
    kw = dict(fuse_merge=mode != "merge_kernel", fuse_steps=mode == "single_launch")
    plan = tb.ChunkAttnPlan(s, q, k, v, w.mask_mode, **kw)
    plan.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.run()
    for rep in range(3):
        q.copy_(torch.roll(q, shifts=rep + 1, dims=0))          # eager work between the replays: new inputs
        eager_out, eager_lse = tb.tasp_chunk_attn(q, k, v, s, w.mask_mode, **kw)
        torch.cuda.synchronize()
        plan.out.zero_()
        plan.lse.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(plan.out, eager_out) and torch.equal(plan.lse, eager_lse), (mode, rep)
