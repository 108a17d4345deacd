"""Pins for oracle/attention.py.  The dense definition is checked against library routines it does
not use (scipy softmax / logsumexp), against pure-Python loops on tiny inputs and against closed
forms; the step-by-step evaluation of Algorithm 3 is checked against the dense one (the
blockwise-merge identity), which also proves that schedule, ranges and mask visit every visible key
exactly once."""
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import attention as att
from oracle import schedule as sch


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- the definition itself
def test_dense_matches_library_softmax():
    S, d, R = 97, 16, 9
    q, k, v = rand((R, d), 1), rand((S, d), 2), rand((S, d), 3)
    pos = np.arange(R) * 7 + 3
    for causal in (False, True):
        out, lse = att.dense_rows(q, pos, k, v, causal)
        for r in range(R):
            nvis = pos[r] + 1 if causal else S
            s = k[:nvis] @ q[r] / math.sqrt(d)
            assert abs(lse[r] - logsumexp(s)) < 1e-12
            np.testing.assert_allclose(out[r], softmax(s) @ v[:nvis], rtol=0, atol=1e-13)


def test_dense_matches_pure_python_loops():
    S, d = 11, 3
    q, k, v = rand((2, d), 4), rand((S, d), 5), rand((S, d), 6)
    pos = [4, 10]
    out, lse = att.dense_rows(q, pos, k, v, True)
    for r in range(2):
        scores = []
        for t in range(S):
            if t <= pos[r]:                                   # reading A2
                scores.append(sum(q[r][c] * k[t][c] for c in range(d)) / math.sqrt(d))
        den = sum(math.exp(x) for x in scores)
        assert abs(lse[r] - math.log(den)) < 1e-12
        for c in range(d):
            ref = sum(math.exp(x) / den * v[t][c] for t, x in enumerate(scores))
            assert abs(out[r][c] - ref) < 1e-12


def test_closed_forms():
    S, d = 64, 8
    q, v = rand((5, d), 7), rand((S, d), 8)
    pos = np.array([0, 1, 17, 40, 63])
    k0 = np.zeros((S, d))
    out, lse = att.dense_rows(q, pos, k0, v, False)
    np.testing.assert_allclose(lse, math.log(S), atol=1e-13)              # ln(#visible)
    np.testing.assert_allclose(out, np.tile(v.mean(0), (5, 1)), atol=1e-13)
    out, lse = att.dense_rows(q, pos, k0, v, True)
    np.testing.assert_allclose(lse, np.log(pos + 1), atol=1e-13)          # ln(p+1): pins reading A2
    for r, p in enumerate(pos):
        np.testing.assert_allclose(out[r], v[: p + 1].mean(0), atol=1e-13)
    k = rand((S, d), 9)
    vc = np.full((S, d), 2.5)
    out, _ = att.dense_rows(q, pos, k, vc, True)
    np.testing.assert_allclose(out, 2.5, atol=1e-13)                      # V constant => O constant
    kk = k.copy()
    kk[13] = 200.0 * q[3] / np.linalg.norm(q[3])                          # one dominant key
    out, lse = att.dense_rows(q[3:4], pos[3:4], kk, v, True)
    np.testing.assert_allclose(out[0], v[13], atol=1e-9)
    assert abs(lse[0] - 200.0 * np.linalg.norm(q[3]) / math.sqrt(d)) < 1e-9


def test_scale_reading():
    """Reading A1: doubling d by zero padding changes the default scale by sqrt(2)."""
    S, d = 20, 4
    q, k, v = rand((1, d), 10), rand((S, d), 11), rand((S, d), 12)
    _, lse = att.dense_rows(q, [S - 1], k, v, False)
    assert abs(lse[0] - logsumexp(k @ q[0] / 2.0)) < 1e-13
    _, lse2 = att.dense_rows(q, [S - 1], k, v, False, scale=1.0)
    assert abs(lse2[0] - logsumexp(k @ q[0])) < 1e-13


# ---------------------------------------------------------------- update_out_lse (reading A4)
def test_merge_equals_softmax_over_the_union():
    d = 5
    q = rand((1, d), 13)[0]
    k, v = rand((30, d), 14), rand((30, d), 15)
    a = list(range(0, 12))
    b = list(range(12, 30))
    oa, la = att.partial_over_tokens(q, 99, k, v, a, False, 0.7)
    ob, lb = att.partial_over_tokens(q, 99, k, v, b, False, 0.7)
    o, l = att.lse_merge(oa[None], np.array([la]), ob[None], np.array([lb]))
    s = k @ q * 0.7
    assert abs(l[0] - logsumexp(s)) < 1e-13
    np.testing.assert_allclose(o[0], softmax(s) @ v, atol=1e-13)
    # commutative
    o2, l2 = att.lse_merge(ob[None], np.array([lb]), oa[None], np.array([la]))
    np.testing.assert_allclose(o2, o, atol=1e-15)
    np.testing.assert_allclose(l2, l, atol=1e-15)


def test_merge_with_empty_partials():
    d = 4
    o = rand((3, d), 16)
    l = np.array([0.3, -2.0, 5.0])
    z = np.zeros((3, d))
    ninf = np.full(3, -np.inf)
    o1, l1 = att.lse_merge(o, l, z, ninf)
    np.testing.assert_array_equal(o1, o)
    np.testing.assert_array_equal(l1, l)
    o2, l2 = att.lse_merge(z, ninf, o, l)
    np.testing.assert_array_equal(o2, o)
    np.testing.assert_array_equal(l2, l)
    o3, l3 = att.lse_merge(z, ninf, z, ninf)
    assert np.all(o3 == 0) and np.all(np.isneginf(l3))
    # extreme gap: the small side vanishes, no NaN
    o4, l4 = att.lse_merge(o, l, o + 1, l - 1e4)
    assert np.all(np.isfinite(o4))
    np.testing.assert_allclose(o4, o, atol=1e-300)
    np.testing.assert_allclose(l4, l, atol=0)


def test_merge_many_equals_softmax_over_the_union_and_the_fold():
    """N partials over disjoint key sets: the one-pass form equals the unsplit softmax (library
    logsumexp / softmax) and the left fold of the pairwise update, in any order of the partials."""
    d = 6
    q = rand((1, d), 21)[0]
    k, v = rand((47, d), 22), rand((47, d), 23)
    cuts = [0, 5, 6, 19, 19, 30, 47]            # one empty set among them
    outs, lses = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        o, l = att.partial_over_tokens(q, 99, k, v, list(range(a, b)), False, 0.9)
        outs.append(o[None])
        lses.append(np.array([l]))
    assert np.isneginf(lses[3][0])
    o, l = att.lse_merge_many(outs, lses)
    s = k @ q * 0.9
    assert abs(l[0] - logsumexp(s)) < 1e-13
    np.testing.assert_allclose(o[0], softmax(s) @ v, atol=1e-13)
    fo, fl = outs[0], lses[0]
    for po, pl in zip(outs[1:], lses[1:]):
        fo, fl = att.lse_merge(fo, fl, po, pl)
    np.testing.assert_allclose(o, fo, atol=1e-13)
    np.testing.assert_allclose(l, fl, atol=1e-13)
    perm = [4, 0, 5, 2, 3, 1]
    o2, l2 = att.lse_merge_many([outs[i] for i in perm], [lses[i] for i in perm])
    np.testing.assert_allclose(o2, o, atol=1e-13)
    np.testing.assert_allclose(l2, l, atol=1e-13)


def test_merge_many_degenerate_cases():
    d = 4
    o = rand((3, d), 24)
    l = np.array([0.3, -2.0, 5.0])
    z = np.zeros((3, d))
    ninf = np.full(3, -np.inf)
    o1, l1 = att.lse_merge_many([o], [l])                       # one partial: unchanged
    np.testing.assert_array_equal(o1, o)
    np.testing.assert_array_equal(l1, l)
    o2, l2 = att.lse_merge_many([z, o, z], [ninf, l, ninf])     # empty partials contribute nothing
    np.testing.assert_array_equal(o2, o)
    np.testing.assert_array_equal(l2, l)
    o3, l3 = att.lse_merge_many([z, z], [ninf, ninf])
    assert np.all(o3 == 0) and np.all(np.isneginf(l3))
    # two equal partials: lse grows by ln 2, out unchanged
    o4, l4 = att.lse_merge_many([o, o], [l, l])
    np.testing.assert_allclose(o4, o, atol=1e-15)
    np.testing.assert_allclose(l4, l + math.log(2.0), atol=1e-15)


# ---------------------------------------------------------------- Algorithm 3 == dense attention
TINY = [(4, 24, 2, 1), (8, 112, 2, 2), (8, 224, 4, 2), (12, 264, 1, 1)]


@pytest.mark.parametrize("n,S,Hq,Hkv", TINY)
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_blockwise_merge_identity_all_ranks(n, S, Hq, Hkv, mode):
    d = 8
    k = rand((S, Hkv, d), 100 + n)
    v = rand((S, Hkv, d), 200 + n)
    ranks = range(n) if n <= 8 else (0, 5, n - 1)
    for rank in ranks:
        pos = sch.local_positions(n, rank, S, mode)
        q = rand((len(pos), Hq, d), 300 + rank)
        for h in range(Hq):
            g = h * Hkv // Hq                                     # reading A3
            ref_o, ref_l = att.dense_rows(q[:, h], pos, k[:, g], v[:, g], mode == sch.ZIGZAG_CAUSAL)
            o, l, partials = att.stepwise_rows(q[:, h], pos, k[:, g], v[:, g], n, rank, mode)
            np.testing.assert_allclose(o, ref_o, rtol=0, atol=1e-12)
            np.testing.assert_allclose(l, ref_l, rtol=0, atol=1e-12)
            assert len(partials) == n
            assert np.all(np.isfinite(l))                         # every row sees itself at step 0


@pytest.mark.parametrize("m,u,S", [(4, 2, 112), (2, 3, 60), (8, 2, 160)])
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_blockwise_merge_identity_multinode_rings(m, u, S, mode):
    """The same identity over the m rings of the (m-K_m-m)^u scheme (m sub-chunks per chunk)."""
    n, d = m * u, 8
    rings = sch.multinode_rings(m, u)
    k, v = rand((S, d), 400 + n), rand((S, d), 500 + n)
    for rank in (0, m - 1, n - 1):
        pos = sch.local_positions(n, rank, S, mode)
        q = rand((len(pos), d), 600 + rank)
        ref_o, ref_l = att.dense_rows(q, pos, k, v, mode == sch.ZIGZAG_CAUSAL)
        o, l, partials = att.stepwise_rows(q, pos, k, v, n, rank, mode, looping=rings)
        np.testing.assert_allclose(o, ref_o, rtol=0, atol=1e-12)
        np.testing.assert_allclose(l, ref_l, rtol=0, atol=1e-12)
        assert len(partials) == n


def test_step_order_does_not_matter():
    n, S, d = 8, 112, 8
    rank = 3
    mode = sch.ZIGZAG_CAUSAL
    k, v = rand((S, d), 21), rand((S, d), 22)
    pos = sch.local_positions(n, rank, S, mode)
    q = rand((len(pos), d), 23)
    o, l, _ = att.stepwise_rows(q, pos, k, v, n, rank, mode)
    perm = list(np.random.default_rng(5).permutation(n))
    o2, l2, _ = att.stepwise_rows(q, pos, k, v, n, rank, mode, step_order=perm)
    np.testing.assert_allclose(o2, o, atol=1e-12)
    np.testing.assert_allclose(l2, l, atol=1e-12)


def test_first_half_rows_see_nothing_from_higher_ranks():
    """Sec. 3.2.3: when src > r only the second half of the queries has work."""
    n, S, d, rank = 8, 112, 4, 2
    mode = sch.ZIGZAG_CAUSAL
    H = S // (2 * n)
    k, v = rand((S, d), 31), rand((S, d), 32)
    pos = sch.local_positions(n, rank, S, mode)
    q = rand((len(pos), d), 33)
    rings = sch.hamilton_rings(n)
    arrival = sch.arrival_table(rings, rank)
    _, _, partials = att.stepwise_rows(q, pos, k, v, n, rank, mode)
    for s in range(1, n):
        if all(src > rank for src in arrival[s]):
            assert np.all(np.isneginf(partials[s][1][:H]))
        assert np.all(np.isfinite(partials[s][1][H:]))


def test_identity_detects_planted_schedule_mistakes(monkeypatch):
    n, S, d, rank = 8, 112, 4, 5
    mode = sch.ZIGZAG_CAUSAL
    k, v = rand((S, d), 41), rand((S, d), 42)
    pos = sch.local_positions(n, rank, S, mode)
    q = rand((len(pos), d), 43)
    ref_o, ref_l = att.dense_rows(q, pos, k, v, True)

    real = sch.subchunk_ranges

    def no_mirror(n_, S_, mode_, ring, src, n_rings=None):            # drop eq. (6)
        return real(n_, S_, mode_, ring, src)[:1]
    monkeypatch.setattr(sch, "subchunk_ranges", no_mirror)
    o, l, _ = att.stepwise_rows(q, pos, k, v, n, rank, mode)
    assert np.max(np.abs(l - ref_l)) > 1e-3
    monkeypatch.setattr(sch, "subchunk_ranges", real)

    real_arr = sch.arrival_table

    def stale(looping, r):                              # one step delivered twice
        t = real_arr(looping, r)
        t[3] = t[2]
        return t
    monkeypatch.setattr(sch, "arrival_table", stale)
    o, l, _ = att.stepwise_rows(q, pos, k, v, n, rank, mode)
    assert np.max(np.abs(l - ref_l)) > 1e-3


def test_flop_counts():
    """4 d Hq pairs; zig-zag pairs have the closed form 2 n H^2 + H."""
    assert att.attention_flops(4, 0, 1024, sch.FULL, 4, 64) == 4 * 64 * 4 * 256 * 1024
    n, S = 8, 131072
    H = S // (2 * n)
    assert att.attention_flops(n, 3, S, sch.ZIGZAG_CAUSAL, 32, 128) == 4 * 128 * 32 * (2 * n * H * H + H)
    assert 2 * n * H * H + H == 1073750016
    for r in range(n):                                  # same work on every rank
        assert att.attention_flops(n, r, S, sch.ZIGZAG_CAUSAL, 1, 1) == 4 * (2 * n * H * H + H)
