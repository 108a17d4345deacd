"""Oracle: one rank's attention, dense and step by step, in fp64 (test infrastructure).

TASP changes only how KV blocks travel (Sec. 3.2.2: accessibility and zero-copy), so the result a
rank must reach is plain attention of its local queries over the whole sequence.  ``dense_rows`` is
that definition written out.  ``stepwise_rows`` follows the forward pass of Algorithm 3 for one rank:
for every step take the sub-chunks that the schedule delivers, attend to their concatenation, and
fold the partial (output, lse) into the running pair (``update_out_lse``).  The two must agree; that
is the blockwise-merge identity the tests check.

Readings (the paper is silent on each; tests/test_oracle_attention.py pins them):
  A1  scores are scaled by 1/sqrt(d); lse is the natural-log sum-exp of the scaled scores.
  A2  causal: key at global position t is visible to the query at global position p iff t <= p.
  A3  query head h reads KV head h * Hkv // Hq (grouped-query attention).
  A4  update_out_lse: lse' = log(e^lse + e^lse_s); out' = e^(lse-lse') out + e^(lse_s-lse') out_s.
      A partial that saw no key has lse = -inf and out = 0 and leaves the running pair unchanged.
  A5  inside a step the sub-chunks are concatenated in ring order (Algorithm 3).
"""
import math

import numpy as np

from . import schedule as sch


def dense_rows(q_rows, positions, k, v, causal, scale=None):
    """softmax(q k^T * scale) v for a few query rows of ONE head.

    q_rows [R, d], positions [R] (global position of each row), k, v [S, d] (the KV head this query
    head reads, natural token order).  Returns (out [R, d], lse [R]) in fp64.
    """
    q = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    positions = np.asarray(positions, dtype=np.int64)
    R, d = q.shape
    S = k.shape[0]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    out = np.zeros((R, d))
    lse = np.full((R,), -np.inf)
    block = max(1, (1 << 25) // S)               # rows per pass, only to bound memory
    key_pos = np.arange(S, dtype=np.int64)
    for r0 in range(0, R, block):
        r1 = min(R, r0 + block)
        s = (q[r0:r1] @ k.T) * scale                                  # [rows, S]
        if causal:
            s = np.where(key_pos[None, :] <= positions[r0:r1, None], s, -np.inf)
        mx = s.max(axis=1, keepdims=True)
        e = np.exp(s - mx)
        den = e.sum(axis=1, keepdims=True)
        lse[r0:r1] = (mx + np.log(den))[:, 0]
        out[r0:r1] = (e / den) @ v
    return out, lse


def partial_over_tokens(q_row, position, k, v, tokens, causal, scale):
    """(out, lse) of one query row over an explicit list of global key positions (one step's
    concatenation).  Keys hidden by the causal rule are dropped; an empty set gives (0, -inf)."""
    tokens = np.asarray(tokens, dtype=np.int64)
    if causal:
        tokens = tokens[tokens <= position]
    d = q_row.shape[0]
    if tokens.size == 0:
        return np.zeros(d), -np.inf
    s = (k[tokens] @ q_row) * scale
    mx = s.max()
    e = np.exp(s - mx)
    den = e.sum()
    return (e / den) @ v[tokens], mx + math.log(den)


def lse_merge(out_a, lse_a, out_b, lse_b):
    """update_out_lse (reading A4) for arrays of rows: out_* [..., d], lse_* [...]."""
    out_a = np.asarray(out_a, dtype=np.float64)
    out_b = np.asarray(out_b, dtype=np.float64)
    lse_a = np.asarray(lse_a, dtype=np.float64)
    lse_b = np.asarray(lse_b, dtype=np.float64)
    mx = np.maximum(lse_a, lse_b)
    safe = np.where(np.isfinite(mx), mx, 0.0)
    with np.errstate(divide="ignore"):
        lse = safe + np.log(np.exp(lse_a - safe) + np.exp(lse_b - safe))
    lse = np.where(np.isfinite(mx), lse, -np.inf)
    ref = np.where(np.isfinite(lse), lse, 0.0)
    wa = np.exp(lse_a - ref)
    wb = np.exp(lse_b - ref)
    return wa[..., None] * out_a + wb[..., None] * out_b, lse


def lse_merge_many(outs, lses):
    """All partial pairs of a row at once: lse = log sum_i exp(lse_i), out = sum_i exp(lse_i - lse) out_i.

    Algorithm 3 folds update_out_lse over the steps one at a time; this is the same quantity written
    out for N partials (the fold telescopes to it).  outs: sequence of [..., d]; lses: sequence of
    [...].  Partials with lse = -inf contribute nothing; if all are -inf the result is (0, -inf).
    """
    outs = [np.asarray(o, dtype=np.float64) for o in outs]
    lses = [np.asarray(l, dtype=np.float64) for l in lses]
    stack = np.stack(lses, axis=0)
    mx = np.max(stack, axis=0)
    safe = np.where(np.isfinite(mx), mx, 0.0)
    den = np.sum(np.exp(stack - safe), axis=0)
    with np.errstate(divide="ignore"):
        lse = np.where(np.isfinite(mx), safe + np.log(den), -np.inf)
    ref = np.where(np.isfinite(lse), lse, 0.0)
    out = np.zeros_like(outs[0])
    for o, l in zip(outs, lses):
        out = out + np.exp(l - ref)[..., None] * o
    return out, lse


def step_tokens(n, rank, S, mask_mode, looping, step):
    """Global key positions a rank holds at `step`, concatenated in ring order (reading A5)."""
    toks = []
    arrival = sch.arrival_table(looping, rank)[step]
    for ring, src in enumerate(arrival):
        for a, b in sch.subchunk_ranges(n, S, mask_mode, ring, src, n_rings=len(looping)):
            toks.extend(range(a, b))
    return toks


def stepwise_rows(q_rows, positions, k, v, n, rank, mask_mode, step_order=None, scale=None, looping=None):
    """Algorithm 3 for a few local rows of one head: N partials folded left to right.

    Returns (out, lse, partials) where partials[s] = (out_s, lse_s) of every step.
    """
    q = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    R, d = q.shape
    S = k.shape[0]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    causal = mask_mode == sch.ZIGZAG_CAUSAL
    looping = sch.hamilton_rings(n) if looping is None else looping      # any ring table over the n ranks
    order = list(range(n)) if step_order is None else list(step_order)
    out = np.zeros((R, d))
    lse = np.full((R,), -np.inf)
    partials = []
    for s in order:
        toks = step_tokens(n, rank, S, mask_mode, looping, s)
        o_s = np.zeros((R, d))
        l_s = np.full((R,), -np.inf)
        for r in range(R):
            o_s[r], l_s[r] = partial_over_tokens(q[r], int(positions[r]), k, v, toks, causal, scale)
        partials.append((o_s, l_s))
        out, lse = lse_merge(out, lse, o_s, l_s)
    return out, lse, partials


def attention_flops(n, rank, S, mask_mode, Hq, d):
    """4 * d * Hq * (number of visible (query, key) pairs) for one rank."""
    pos = sch.local_positions(n, rank, S, mask_mode)
    if mask_mode == sch.ZIGZAG_CAUSAL:
        pairs = sum(p + 1 for p in pos)
    else:
        pairs = len(pos) * S
    return 4 * d * Hq * pairs
