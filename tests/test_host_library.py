"""CPU-side tests of libtasp.so: the library loads, exports what include/tasp.h declares, and its
integer outputs (rings, routing tables, arrival order, sub-chunk ranges, per-step segment lists) are
bit-exact with the oracle.  No compute entry point is called here."""
import ctypes as C
import os
import re

import pytest

from oracle import attention as att
from oracle import schedule as sch
from paper_2509_26541_amd import binding as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NS = [4, 8, 12, 16, 20, 24, 32, 48, 64]


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "tasp.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(tasp_[a-z0-9_]+)\s*\(", text)))
    assert declared == sorted(tb.EXPORTS)
    raw = C.CDLL(tb.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


@pytest.mark.parametrize("m,u", [(2, 2), (4, 2), (8, 2), (8, 3), (6, 5), (16, 2), (32, 2), (8, 8)])
def test_multinode_schedule_bit_exact_all_ranks(m, u):
    rings = sch.multinode_rings(m, u)
    n = m * u
    out_m, in_m = sch.out_mapping(rings), sch.in_mapping(rings)
    for rank in range(n):
        s = tb.tasp_schedule_multinode(m, u, rank)
        assert (s.n_ranks, s.rank, s.n_rings, s.max_arc_load) == (n, rank, m, 1)
        assert s.rings.tolist() == rings
        assert s.out_mapping.tolist() == out_m
        assert s.in_mapping.tolist() == in_m
        assert s.arrival.tolist() == sch.arrival_table(rings, rank)
    S = 2 * n * 37
    s = tb.tasp_schedule_multinode(m, u, n - 1)
    for mode in (sch.FULL, sch.ZIGZAG_CAUSAL):
        for ring in range(m):
            for src in (0, n // 2, n - 1):
                assert s.subchunk_ranges(S, mode, ring, src) == sch.subchunk_ranges(n, S, mode, ring, src, n_rings=m)
    h = C.c_void_p()
    for args, code in [((3, 2, 0), tb.EUNSUPPORTED_N), ((8, 1, 0), tb.EUNSUPPORTED_N), ((0, 2, 0), tb.EINVAL),
                       ((8, 2, 16), tb.EINVAL), ((8, 2, -1), tb.EINVAL), ((64, 128, 0), tb.EUNSUPPORTED_N)]:
        assert tb.lib.tasp_schedule_create_multinode(*args, C.byref(h)) == code and not h.value
    assert tb.lib.tasp_schedule_create_multinode(8, 2, 0, None) == tb.EINVAL


@pytest.mark.parametrize("n", NS)
def test_schedule_bit_exact_all_ranks(n):
    rings = sch.hamilton_rings(n)
    out_m, in_m = sch.out_mapping(rings), sch.in_mapping(rings)
    for rank in range(n):
        s = tb.tasp_schedule(n, rank)
        assert (s.n_ranks, s.rank, s.n_rings) == (n, rank, n - 1)
        assert s.rings.tolist() == rings
        assert s.out_mapping.tolist() == out_m
        assert s.in_mapping.tolist() == in_m
        assert s.arrival.tolist() == sch.arrival_table(rings, rank)
        assert s.max_arc_load == max(sch.arc_loads(rings).values()) == (2 if n == 4 else 1)


@pytest.mark.parametrize("n,S", [(4, 24), (4, 1024), (8, 112), (8, 131072), (16, 524288), (8, 1048576), (12, 264)])
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_subchunk_ranges_bit_exact(n, S, mode):
    s = tb.tasp_schedule(n, 1)
    for src in range(n):
        for ring in range(n - 1):
            assert s.subchunk_ranges(S, mode, ring, src) == sch.subchunk_ranges(n, S, mode, ring, src)


def expand(segs):
    return [t for a, b, _ in segs for t in range(a, b)]


@pytest.mark.parametrize("n,S", [(4, 24), (8, 112), (8, 2048), (12, 264), (16, 544)])
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_step_segments_against_oracle(n, S, mode):
    """Expanded in order, the segments of (step, block) are the oracle's concatenation for that step
    minus the keys no row of the block may see; the diag flag marks segments some row sees in part."""
    from oracle import attention as att
    rings = sch.hamilton_rings(n)
    for rank in range(n):
        s = tb.tasp_schedule(n, rank)
        pos = sch.local_positions(n, rank, S, mode)
        blocks = [pos] if mode == sch.FULL else [pos[: len(pos) // 2], pos[len(pos) // 2:]]
        for step in range(n):
            toks = att.step_tokens(n, rank, S, mode, rings, step)
            for qb, rows in enumerate(blocks):
                segs = s.step_segments(S, mode, step, qb)
                want = toks if mode == sch.FULL else [t for t in toks if t <= rows[-1]]
                assert expand(segs) == want
                for a, b, diag in segs:
                    assert a < b
                    assert diag == (1 if (mode == sch.ZIGZAG_CAUSAL and b - 1 > rows[0]) else 0)
                for (a0, b0, d0), (a1, b1, d1) in zip(segs, segs[1:]):
                    assert not (b0 == a1 and d0 == d1)          # neighbours were joined


@pytest.mark.parametrize("m,u,S", [(4, 2, 112), (8, 2, 480), (2, 3, 60)])
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_step_segments_multinode_against_oracle(m, u, S, mode):
    from oracle import attention as att
    n = m * u
    rings = sch.multinode_rings(m, u)
    for rank in range(n):
        s = tb.tasp_schedule_multinode(m, u, rank)
        pos = sch.local_positions(n, rank, S, mode)
        blocks = [pos] if mode == sch.FULL else [pos[: len(pos) // 2], pos[len(pos) // 2:]]
        for step in range(n):
            toks = att.step_tokens(n, rank, S, mode, rings, step)
            for qb, rows in enumerate(blocks):
                segs = s.step_segments(S, mode, step, qb)
                want = toks if mode == sch.FULL else [t for t in toks if t <= rows[-1]]
                assert expand(segs) == want


def test_zigzag_classification_matches_the_load_balance_argument():
    """Sec. 3.2.3: src < r: both halves of the queries see piece [0] only; src > r: only the second
    half sees anything, and it sees both pieces; src == r (step 0): the diagonal blocks."""
    n, S, rank = 8, 131072, 3
    H = S // (2 * n)
    s = tb.tasp_schedule(n, rank)
    for step in range(n):
        lo = s.step_segments(S, sch.ZIGZAG_CAUSAL, step, 0)
        hi = s.step_segments(S, sch.ZIGZAG_CAUSAL, step, 1)
        keys_lo = sum(b - a for a, b, _ in lo)
        keys_hi = sum(b - a for a, b, _ in hi)
        srcs = s.arrival[step].tolist()
        exp_lo = exp_hi = 0
        for ring, src in enumerate(srcs):
            (a0, b0), (a1, b1) = sch.subchunk_ranges(n, S, sch.ZIGZAG_CAUSAL, ring, src)
            if src < rank:
                exp_lo += b0 - a0
                exp_hi += b0 - a0
            elif src > rank:
                exp_hi += (b0 - a0) + (b1 - a1)
            else:
                exp_lo += b0 - a0
                exp_hi += (b0 - a0) + (b1 - a1)
        assert (keys_lo, keys_hi) == (exp_lo, exp_hi)
        if step == 0:
            assert lo == [(rank * H, (rank + 1) * H, 1)]
            assert all(d == 1 for a, b, d in hi if a >= S // 2) and all(d == 0 for a, b, d in hi if a < S // 2)
        else:
            assert all(d == 0 for _, _, d in lo + hi)


def test_ring_order_segments():
    n, S, rank = 8, 2048, 5
    s = tb.tasp_schedule(n, rank)
    L, H = S // n, S // (2 * n)
    for step in range(n):
        src = (rank - step) % n
        assert s.step_segments(S, sch.FULL, step, 0, order=tb.ORDER_RING) == [(src * L, (src + 1) * L, 0)]
        hi = s.step_segments(S, sch.ZIGZAG_CAUSAL, step, 1, order=tb.ORDER_RING)
        lo = s.step_segments(S, sch.ZIGZAG_CAUSAL, step, 0, order=tb.ORDER_RING)
        if src < rank:
            assert lo == hi == [(src * H, (src + 1) * H, 0)]
        elif src > rank:
            both = [(src * H, (src + 1) * H, 0), (S - (src + 1) * H, S - src * H, 0)]
            if src == n - 1:                         # the two halves of the last rank touch
                both = [(src * H, S - src * H, 0)]
            assert lo == [] and hi == both
        else:
            assert lo == [(src * H, (src + 1) * H, 1)]
            assert hi == [(src * H, (src + 1) * H, 0), (S - (src + 1) * H, S - src * H, 1)]


def test_error_codes():
    h = C.c_void_p()
    assert tb.lib.tasp_schedule_create(8, 0, None) == tb.EINVAL
    for n, r, code in [(1, 0, tb.EINVAL), (8, 8, tb.EINVAL), (8, -1, tb.EINVAL), (6, 0, tb.EUNSUPPORTED_N),
                       (10, 0, tb.EUNSUPPORTED_N), (5, 0, tb.EUNSUPPORTED_N), (7, 3, tb.EUNSUPPORTED_N)]:
        assert tb.lib.tasp_schedule_create(n, r, C.byref(h)) == code
        assert not h.value
    s = tb.tasp_schedule(8, 0)
    r = (C.c_int64 * 4)()
    cnt = C.c_int32()
    assert tb.lib.tasp_subchunk_ranges(s.handle, 100, 0, 0, 0, r, C.byref(cnt)) == tb.EINVAL      # 100 % 8
    assert tb.lib.tasp_subchunk_ranges(s.handle, 104, 1, 0, 0, r, C.byref(cnt)) == tb.EINVAL      # 104 % 16
    assert tb.lib.tasp_subchunk_ranges(s.handle, 128, 0, 7, 0, r, C.byref(cnt)) == tb.EINVAL      # ring
    assert tb.lib.tasp_subchunk_ranges(s.handle, 128, 2, 0, 0, r, C.byref(cnt)) == tb.EINVAL      # mode
    assert tb.lib.tasp_subchunk_ranges(None, 128, 0, 0, 0, r, C.byref(cnt)) == tb.EINVAL
    with pytest.raises(tb.TaspError):
        s.step_segments(128, 0, 8, 0)
    with pytest.raises(tb.TaspError):
        s.step_segments(128, 0, 0, 1)            # FULL has one query block
    assert tb.lib.tasp_schedule_n_ranks(None) == 0 and not tb.lib.tasp_schedule_rings(None)
    for code in range(-8, 1):
        assert tb.strerror(code)
    # argument checks of the compute entry points that return before any HIP call
    a = tb.AttnArgs()
    assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EINVAL
    assert tb.lib.tasp_chunk_attn(None, C.byref(a), None) == tb.EINVAL
    a.q = a.k = a.v = 4096
    a.out = a.lse = 4096
    a.S, a.Hq, a.Hkv, a.d, a.dtype, a.mask_mode = 1024, 4, 4, 64, tb.DTYPE_FP32, tb.MASK_FULL
    assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EWORKSPACE
    a.d = 96
    assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EUNSUPPORTED_SHAPE
    a.d, a.Hq = 64, 6
    assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EINVAL
    a.Hq, a.q = 4, 4100
    assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EALIGN
    a.q, a.S = 4096, 1001
    assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EINVAL
    assert tb.lib.tasp_lse_merge(None, None, None, None, 4, 2, 64, None) == tb.EINVAL
    assert tb.lib.tasp_lse_merge(4096, 4096, 4096, 4096, 4, 2, 24, None) == tb.EUNSUPPORTED_SHAPE
    assert tb.lib.tasp_lse_merge(4096, 4096, 4104, 4096, 4, 2, 64, None) == tb.EALIGN
    assert tb.lib.tasp_lse_merge(None, None, None, None, 0, 2, 64, None) == tb.OK
    two = (C.c_void_p * 2)(4096, 8192)
    odd = (C.c_void_p * 2)(4096, 8200)
    hole = (C.c_void_p * 2)(4096, None)
    many = tb.lib.tasp_lse_merge_many
    assert many(4096, 4096, two, two, 0, 4, 2, 64, None) == tb.EINVAL                    # no partial
    assert many(4096, 4096, two, two, 65, 4, 2, 64, None) == tb.EINVAL                   # more than the maximum
    assert many(4096, 4096, None, two, 2, 4, 2, 64, None) == tb.EINVAL
    assert many(None, 4096, two, two, 2, 4, 2, 64, None) == tb.EINVAL
    assert many(4096, 4096, hole, two, 2, 4, 2, 64, None) == tb.EINVAL
    assert many(4096, 4096, two, two, 2, 4, 2, 48, None) == tb.EUNSUPPORTED_SHAPE
    assert many(4096, 4096, odd, two, 2, 4, 2, 64, None) == tb.EALIGN
    assert many(None, None, None, None, 2, 0, 2, 64, None) == tb.OK                      # no rows: nothing to do
    assert tb.lib.tasp_calibration_mfma(0, None, None) == tb.EINVAL
    assert tb.lib.tasp_calibration_mfma((1 << 20) + 1, None, None) == tb.EINVAL


def test_flops_and_workspace():
    from oracle import attention as att
    for n, rank, S, mode, Hq, Hkv, d, dt in [(4, 0, 1024, 0, 4, 4, 64, 0), (8, 3, 131072, 1, 32, 8, 128, 1),
                                             (8, 0, 262144, 0, 32, 8, 128, 1), (16, 5, 524288, 1, 64, 8, 128, 1),
                                             (8, 7, 1048576, 1, 32, 8, 128, 1)]:
        s = tb.tasp_schedule(n, rank)
        a = tb.AttnArgs()
        a.S, a.Hq, a.Hkv, a.d, a.dtype, a.mask_mode = S, Hq, Hkv, d, dt, mode
        assert tb.lib.tasp_chunk_attn_flops(s.handle, C.byref(a)) == float(att.attention_flops(n, rank, S, mode, Hq, d))
        L = S // n
        o, l = L * Hq * d * 4, L * Hq * 4
        a.fuse_merge = 0
        assert tb.lib.tasp_chunk_attn_workspace_bytes(s.handle, C.byref(a)) == (o if dt else 0) + o + l
        a.fuse_merge = 1
        assert tb.lib.tasp_chunk_attn_workspace_bytes(s.handle, C.byref(a)) == (o if dt else 0)
        # a batch of B sequences is B times the work and B times the buffers
        a.batch, a.fuse_merge = 3, 0
        assert tb.lib.tasp_chunk_attn_flops(s.handle, C.byref(a)) == 3 * float(att.attention_flops(n, rank, S, mode, Hq, d))
        assert tb.lib.tasp_chunk_attn_workspace_bytes(s.handle, C.byref(a)) == 3 * ((o if dt else 0) + o + l)
        a.batch = -1
        assert tb.lib.tasp_chunk_attn_workspace_bytes(s.handle, C.byref(a)) == 0
        assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EINVAL
        # all steps in one launch: the running output (bf16 only) and the segment table
        a.batch, a.fuse_steps = 1, 1
        assert tb.lib.tasp_chunk_attn_workspace_bytes(s.handle, C.byref(a)) == (o if dt else 0) + 2 * 2 * 1024 * 4
        a.q = a.k = a.v = a.out = a.lse = 4096
        a.fuse_steps = 2
        assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EINVAL
        a.fuse_steps = 1
        assert tb.lib.tasp_chunk_attn(s.handle, C.byref(a), None) == tb.EWORKSPACE        # both types take the single launch


def test_backward_argument_checks_and_sizes():
    """tasp_chunk_attn_bwd: argument checks that return before any HIP call, workspace size (an fp32 dq,
    the delta vector, partial dk and dv) and the flops convention (2.5 times the forward's)."""
    s = tb.tasp_schedule(8, 3)
    b = tb.AttnBwdArgs()
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EINVAL
    assert tb.lib.tasp_chunk_attn_bwd(None, C.byref(b), None) == tb.EINVAL
    assert tb.lib.tasp_chunk_attn_bwd_profile(s.handle, C.byref(b), None, None) == tb.EINVAL
    b.q = b.k = b.v = 4096
    b.S, b.Hq, b.Hkv, b.d, b.dtype, b.mask_mode = 4096, 8, 2, 128, tb.DTYPE_BF16, tb.MASK_ZIGZAG_CAUSAL
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EINVAL           # out, lse, dout, dq, dk, dv missing
    b.out = b.lse = b.dout = b.dq = b.dk = b.dv = 4096
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EWORKSPACE
    b.d = 96
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EUNSUPPORTED_SHAPE
    b.d, b.dtype = 128, tb.DTYPE_FP32
    assert tb.lib.tasp_chunk_attn_bwd_workspace_bytes(s.handle, C.byref(b)) == (4096 // 8 * 8 * 4 + 255) // 256 * 256   # delta only
    b.dtype, b.dk = tb.DTYPE_BF16, 4104
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EALIGN
    b.dk, b.batch = 4096, -1
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EINVAL
    b.batch = 0
    L = 4096 // 8
    pad = lambda x: (x + 255) // 256 * 256
    # fp32 dq, delta and lse log2(e) (one entry more than rows each) and (grouped heads, step by step)
    # the partial dk and dv of one step per query head
    rows = lambda n: 2 * pad((n + 1) * 4)
    assert tb.lib.tasp_chunk_attn_bwd_workspace_bytes(s.handle, C.byref(b)) == 3 * pad(L * 8 * 128 * 4) + rows(L * 8)
    b.Hkv = 8                                           # one query head per KV head: no partial sums
    assert tb.lib.tasp_chunk_attn_bwd_workspace_bytes(s.handle, C.byref(b)) == pad(L * 8 * 128 * 4) + rows(L * 8)
    b.Hkv = 2
    fwd = att.attention_flops(8, 3, 4096, sch.ZIGZAG_CAUSAL, 8, 128)
    assert tb.lib.tasp_chunk_attn_bwd_flops(s.handle, C.byref(b)) == 2.5 * fwd
    from oracle import attention_bwd as bwd
    assert bwd.attention_bwd_flops(8, 3, 4096, sch.ZIGZAG_CAUSAL, 8, 128) == 2.5 * fwd
    b.batch = 4
    assert tb.lib.tasp_chunk_attn_bwd_workspace_bytes(s.handle, C.byref(b)) == 3 * pad(4 * L * 8 * 128 * 4) + rows(4 * L * 8)
    # bf16: the row arrays are addressed with 32-bit byte offsets, so 2^30 (row, head) pairs are refused
    # (checked after the workspace and before anything is enqueued)
    big = tb.AttnBwdArgs()
    big.q = big.k = big.v = big.out = big.lse = big.dout = big.dq = big.dk = big.dv = big.workspace = 4096
    big.workspace_bytes = 1 << 62
    big.S, big.Hq, big.Hkv, big.d, big.dtype, big.mask_mode, big.batch = 1 << 20, 64, 1, 64, tb.DTYPE_BF16, tb.MASK_ZIGZAG_CAUSAL, 128
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(big), None) == tb.EUNSUPPORTED_SHAPE
    b.fuse_steps = 1                                    # plus the segment table of the single launch
    assert tb.lib.tasp_chunk_attn_bwd_workspace_bytes(s.handle, C.byref(b)) == pad(4 * L * 8 * 128 * 4) + rows(4 * L * 8) + 2 * 2 * 1024 * 4
    b.fuse_steps = 3
    assert tb.lib.tasp_chunk_attn_bwd(s.handle, C.byref(b), None) == tb.EINVAL
    b.fuse_steps = 0
    assert tb.lib.tasp_chunk_attn_bwd_flops(s.handle, C.byref(b)) == 4 * 2.5 * fwd


def test_documented_size_limits_of_the_attention_call():
    """The limits tasp.h states, from both sides, before any HIP call: 32 ranks (62 segments a step)
    pass the shape checks and 36 do not; K/V of exactly 2^32 bytes per tensor pass and one more row of
    tokens does not; S must stay below 2^24 for bf16."""
    a = tb.AttnArgs()
    a.q = a.k = a.v = a.out = a.lse = 4096
    a.Hq, a.Hkv, a.d, a.dtype, a.mask_mode = 8, 8, 128, tb.DTYPE_BF16, tb.MASK_ZIGZAG_CAUSAL
    a.S = 64 * 36
    assert tb.lib.tasp_chunk_attn(tb.tasp_schedule(32, 5).handle, C.byref(a), None) == tb.EWORKSPACE
    a.S = 72 * 36
    assert tb.lib.tasp_chunk_attn(tb.tasp_schedule(36, 5).handle, C.byref(a), None) == tb.EUNSUPPORTED_SHAPE
    s8 = tb.tasp_schedule(8, 0)
    a.S = 1 << 21                                     # x 8 heads x 128 x 2 bytes = 2^32
    assert tb.lib.tasp_chunk_attn(s8.handle, C.byref(a), None) == tb.EWORKSPACE
    a.S = (1 << 21) + 16
    assert tb.lib.tasp_chunk_attn(s8.handle, C.byref(a), None) == tb.EUNSUPPORTED_SHAPE
    a.Hq = a.Hkv = 1
    a.d = 64
    a.S = (1 << 24) - 16
    assert tb.lib.tasp_chunk_attn(s8.handle, C.byref(a), None) == tb.EWORKSPACE
    a.S = 1 << 24
    assert tb.lib.tasp_chunk_attn(s8.handle, C.byref(a), None) == tb.EUNSUPPORTED_SHAPE
    a.S, a.batch = 1024, 65535                       # the most sequences one call takes
    assert tb.lib.tasp_chunk_attn(s8.handle, C.byref(a), None) == tb.EWORKSPACE
    a.batch = 65536
    assert tb.lib.tasp_chunk_attn(s8.handle, C.byref(a), None) == tb.EINVAL
