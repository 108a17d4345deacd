"""Pins for oracle/attention_bwd.py.  The gradient formula is checked against central finite
differences of the forward oracle, against reverse-mode differentiation by a library (torch
autograd over its own softmax), against pure-Python loops on tiny inputs and against closed forms
and invariants; the step-by-step walk in the forward's arrival order is checked against the dense
gradient, which proves that every visible (query, key) pair is visited exactly once."""
import math

import numpy as np
import pytest
import torch

from oracle import attention as att
from oracle import attention_bwd as bwd
from oracle import schedule as sch


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def loss(q, pos, k, v, do, causal):
    out, _ = att.dense_rows(q, pos, k, v, causal)
    return float((do * out).sum())


# ---------------------------------------------------------------- the gradient itself
@pytest.mark.parametrize("causal", [False, True])
def test_grads_match_finite_differences_of_the_forward_oracle(causal):
    S, d, R = 23, 5, 7
    q, k, v, do = rand((R, d), 1), rand((S, d), 2), rand((S, d), 3), rand((R, d), 4)
    pos = np.array([0, 3, 4, 9, 15, 22, 22])
    dq, dk, dv = bwd.dense_grads(q, pos, k, v, do, causal)
    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for idx in np.ndindex(x.shape):
            x0 = x[idx]
            x[idx] = x0 + eps
            up = loss(q, pos, k, v, do, causal)
            x[idx] = x0 - eps
            dn = loss(q, pos, k, v, do, causal)
            x[idx] = x0
            assert abs((up - dn) / (2 * eps) - g[idx]) < 2e-8, (name, idx)


@pytest.mark.parametrize("causal", [False, True])
def test_grads_match_library_autograd(causal):
    S, d, R = 61, 8, 13
    q, k, v, do = rand((R, d), 5), rand((S, d), 6), rand((S, d), 7), rand((R, d), 8)
    pos = np.sort(np.random.default_rng(9).integers(0, S, R))
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    s = tq @ tk.T / math.sqrt(d)
    if causal:
        hidden = torch.arange(S)[None, :] > torch.tensor(pos)[:, None]
        s = s.masked_fill(hidden, float("-inf"))
    out = torch.softmax(s, dim=1) @ tv
    (out * torch.tensor(do)).sum().backward()
    dq, dk, dv = bwd.dense_grads(q, pos, k, v, do, causal)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-13)


def test_grads_match_pure_python_loops():
    """The quotient rule applied term by term: d out_i / d s_ij = p_ij (v_j - out_i)."""
    S, d = 6, 3
    q, k, v, do = rand((2, d), 10), rand((S, d), 11), rand((S, d), 12), rand((2, d), 13)
    pos = [2, 5]
    c = 1 / math.sqrt(d)
    dq_ref = [[0.0] * d for _ in range(2)]
    dk_ref = [[0.0] * d for _ in range(S)]
    dv_ref = [[0.0] * d for _ in range(S)]
    for i in range(2):
        vis = list(range(pos[i] + 1))
        sc = [c * sum(q[i][a] * k[j][a] for a in range(d)) for j in vis]
        z = sum(math.exp(x) for x in sc)
        p = [math.exp(x) / z for x in sc]
        out = [sum(p[n] * v[j][a] for n, j in enumerate(vis)) for a in range(d)]
        for n, j in enumerate(vis):
            dsij = p[n] * sum(do[i][a] * (v[j][a] - out[a]) for a in range(d))
            for a in range(d):
                dq_ref[i][a] += c * dsij * k[j][a]
                dk_ref[j][a] += c * dsij * q[i][a]
                dv_ref[j][a] += p[n] * do[i][a]
    dq, dk, dv = bwd.dense_grads(q, pos, k, v, do, True)
    np.testing.assert_allclose(dq, dq_ref, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dk, dk_ref, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dv, dv_ref, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- closed forms and invariants
def test_single_visible_key():
    """One visible key: out = v_0 whatever q is, so dq = dk = 0 and dv_0 = dout."""
    d = 4
    q, k, v, do = rand((1, d), 14), rand((5, d), 15), rand((5, d), 16), rand((1, d), 17)
    dq, dk, dv = bwd.dense_grads(q, [0], k, v, do, True)
    assert np.abs(dq).max() < 1e-15 and np.abs(dk).max() < 1e-15
    np.testing.assert_allclose(dv[0], do[0], rtol=0, atol=1e-15)
    assert np.all(dv[1:] == 0.0) and np.all(dk[1:] == 0.0)


def test_equal_keys_give_uniform_probabilities():
    """All keys equal: p = 1/S, so dv_j = mean-weighted dout, dq = scale * sum_j ds_ij k = 0 (the
    rows of ds sum to zero and every k_j is the same vector)."""
    S, d, R = 9, 4, 3
    q, do, v = rand((R, d), 18), rand((R, d), 19), rand((S, d), 20)
    k = np.tile(rand((1, d), 21), (S, 1))
    dq, dk, dv = bwd.dense_grads(q, np.arange(R), k, v, do, False)
    assert np.abs(dq).max() < 1e-14
    np.testing.assert_allclose(dv, np.tile(do.sum(0) / S, (S, 1)), rtol=0, atol=1e-14)
    out = v.mean(0)
    want = sum(np.outer((v @ do[i] - do[i] @ out) / S, q[i]) for i in range(R)) / math.sqrt(d)
    np.testing.assert_allclose(dk, want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_invariants(causal):
    """Rows of p sum to one: sum_j dv_j = sum_i dout_i.  Rows of ds sum to zero, and
    sum_j dk_j = scale * sum_i (sum_j ds_ij) q_i, so it is zero too.  Keys no query sees get exactly
    zero.  The gradient is linear in dout."""
    S, d, R = 40, 6, 11
    q, k, v, do = rand((R, d), 22), rand((S, d), 23), rand((S, d), 24), rand((R, d), 25)
    pos = np.sort(np.random.default_rng(26).integers(0, 30, R))
    dq, dk, dv = bwd.dense_grads(q, pos, k, v, do, causal)
    np.testing.assert_allclose(dv.sum(0), do.sum(0), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dk.sum(0), np.zeros(d), rtol=0, atol=1e-13)
    if causal:
        assert np.all(dk[pos.max() + 1:] == 0.0) and np.all(dv[pos.max() + 1:] == 0.0)
    # linearity: zero dout on some rows = those rows removed
    keep = np.array([1, 4, 5, 9])
    do2 = np.zeros_like(do)
    do2[keep] = do[keep]
    dq2, dk2, dv2 = bwd.dense_grads(q, pos, k, v, do2, causal)
    dq3, dk3, dv3 = bwd.dense_grads(q[keep], pos[keep], k, v, do[keep], causal)
    np.testing.assert_allclose(dq2[keep], dq3, rtol=0, atol=1e-14)
    assert np.all(np.delete(dq2, keep, axis=0) == 0.0)
    np.testing.assert_allclose(dk2, dk3, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dv2, dv3, rtol=0, atol=1e-14)


def test_stored_output_only_enters_through_delta():
    """Reading B5: with the exact output passed in, nothing changes; a perturbed stored output changes
    ds by -p * (dout . perturbation) and leaves dv alone."""
    S, d, R = 14, 4, 3
    q, k, v, do = rand((R, d), 70), rand((S, d), 71), rand((S, d), 72), rand((R, d), 73)
    pos = np.arange(R) + 9
    out, lse = att.dense_rows(q, pos, k, v, True)
    base = bwd.dense_grads(q, pos, k, v, do, True)
    same = bwd.dense_grads(q, pos, k, v, do, True, out_rows=out)
    for a, b in zip(base, same):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-15)
    bump = rand((R, d), 74) * 1e-2
    dq2, dk2, dv2 = bwd.dense_grads(q, pos, k, v, do, True, out_rows=out + bump)
    np.testing.assert_allclose(dv2, base[2], rtol=0, atol=1e-15)
    c = 1 / math.sqrt(d)
    s = np.where(np.arange(S)[None] <= pos[:, None], q @ k.T * c, -np.inf)
    p = np.exp(s - lse[:, None])
    shift = -(do * bump).sum(1, keepdims=True) * p                # change of ds
    np.testing.assert_allclose(dq2 - base[0], shift @ k * c, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dk2 - base[1], shift.T @ q * c, rtol=0, atol=1e-14)


def test_shift_of_the_scores_changes_nothing():
    """Softmax is invariant under a per-row shift: adding a constant vector u to every key shifts the
    scores of row i by scale * q_i.u; out, dv and dq's ds stay, so dv is unchanged."""
    S, d, R = 12, 4, 3
    q, k, v, do = rand((R, d), 27), rand((S, d), 28), rand((S, d), 29), rand((R, d), 30)
    _, _, dv0 = bwd.dense_grads(q, np.arange(R), k, v, do, False)
    _, _, dv1 = bwd.dense_grads(q, np.arange(R), k + rand((1, d), 31), v, do, False)
    np.testing.assert_allclose(dv0, dv1, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- the walk in arrival order
CASES = [
    (4, 1, 64, sch.FULL), (4, 2, 64, sch.ZIGZAG_CAUSAL), (8, 3, 176, sch.ZIGZAG_CAUSAL), (8, 0, 120, sch.FULL),
    (8, 7, 16 * 9, sch.ZIGZAG_CAUSAL), (12, 4, 24 * 5, sch.ZIGZAG_CAUSAL),
]


@pytest.mark.parametrize("n,rank,S,mode", CASES)
def test_stepwise_equals_dense(n, rank, S, mode):
    d = 8
    pos = np.asarray(sch.local_positions(n, rank, S, mode))
    rows = np.arange(len(pos))
    q, k, v, do = rand((len(rows), d), 40 + n), rand((S, d), 41), rand((S, d), 42), rand((len(rows), d), 43)
    dq, dk, dv, per_step = bwd.stepwise_grads(q, pos, k, v, do, n, rank, mode)
    dq0, dk0, dv0 = bwd.dense_grads(q, pos, k, v, do, mode == sch.ZIGZAG_CAUSAL)
    np.testing.assert_allclose(dq, dq0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, dk0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, dv0, rtol=0, atol=1e-12)
    # every key is held at exactly one step
    seen = np.concatenate([t for t, _ in per_step])
    assert sorted(seen.tolist()) == list(range(S))


def test_stepwise_on_a_multinode_scheme():
    m, u, S, d = 4, 2, 8 * 2 * 12, 8
    looping = sch.multinode_rings(m, u)
    n = m * u
    for mode in (sch.FULL, sch.ZIGZAG_CAUSAL):
        pos = np.asarray(sch.local_positions(n, 5, S, mode))
        q, k, v, do = rand((len(pos), d), 50), rand((S, d), 51), rand((S, d), 52), rand((len(pos), d), 53)
        dq, dk, dv, _ = bwd.stepwise_grads(q, pos, k, v, do, n, 5, mode, looping=looping)
        dq0, dk0, dv0 = bwd.dense_grads(q, pos, k, v, do, mode == sch.ZIGZAG_CAUSAL)
        for a, b in ((dq, dq0), (dk, dk0), (dv, dv0)):
            np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def test_planted_mistakes_are_caught():
    """A dropped delta term, a transposed product or a wrong sign each break a pin above; here the
    delta term and the scale are planted in a copy of the formula to show the finite-difference pin
    has the resolution to see them."""
    S, d, R = 10, 3, 4
    q, k, v, do = rand((R, d), 60), rand((S, d), 61), rand((S, d), 62), rand((R, d), 63)
    pos = np.arange(R) + 5
    dq, _, _ = bwd.dense_grads(q, pos, k, v, do, True)
    out, lse = att.dense_rows(q, pos, k, v, True)
    c = 1 / math.sqrt(d)
    s = np.where(np.arange(S)[None] <= pos[:, None], q @ k.T * c, -np.inf)
    p = np.exp(s - lse[:, None])
    wrong = (p * (do @ v.T)) @ k * c                     # delta dropped
    assert np.abs(wrong - dq).max() > 1e-3
    eps = 1e-6
    q2 = q.copy(); q2[1, 2] += eps
    q3 = q.copy(); q3[1, 2] -= eps
    fd = (loss(q2, pos, k, v, do, True) - loss(q3, pos, k, v, do, True)) / (2 * eps)
    assert abs(fd - dq[1, 2]) < 1e-8 < abs(fd - wrong[1, 2])


def test_flops_convention():
    assert bwd.attention_bwd_flops(8, 3, 1024, sch.ZIGZAG_CAUSAL, 4, 64) * 2 == att.attention_flops(8, 3, 1024, sch.ZIGZAG_CAUSAL, 4, 64) * 5
