"""Oracle: gradients of one rank's attention, dense and step by step, in fp64 (test infrastructure).

The paper evaluates the forward pass only (Sec. 5.1.2; the backward pass is named as the training
use of the same schedule).  What a rank's backward pass must reach therefore has a plain
definition: the gradient of  loss = sum(dout * out)  where  out = attention(q_local, k, v)  is the
forward result of its local query rows over the whole sequence.  ``dense_grads`` is that gradient
written out with the softmax Jacobian.  ``stepwise_grads`` walks the steps of Algorithm 3 in the
forward's arrival order: the KV sub-chunks a rank holds at a step receive their dk / dv from the
local queries (each key is held at exactly one step, so its gradient is complete after that step),
and dq accumulates over the steps.  The two must agree.

What is returned for k and v is THIS RANK'S contribution (its local query rows only); the sum over
ranks, which travels back along the rings in a distributed run, is not part of this.

Readings (the paper is silent on each; tests/test_oracle_attention_bwd.py pins them):
  B1  the probabilities are recomputed from the FINAL lse of the forward pass:
      p = exp(scale * q.k - lse); nothing per step is kept from the forward.
  B2  delta = sum_d(dout * out) with the final out; ds = p * (dout.v - delta);
      dq = scale * ds k,  dk = scale * ds^T q,  dv = p^T dout.
  B3  grouped-query attention: a KV head receives the sum over the query heads that read it.
  B4  a query row that saw no key (lse = -inf) has p = 0 and contributes nothing.
  B5  the forward output is an INPUT of the backward call (it was stored, in the storage precision);
      ``out_rows`` passes such a stored copy, and delta is then taken from it as B2 says.  Left out,
      the exact output is used, which is the gradient's plain definition.
"""
import math

import numpy as np

from . import attention as att
from . import schedule as sch


def dense_grads(q_rows, positions, k, v, dout_rows, causal, scale=None, out_rows=None):
    """Gradients of sum(dout * softmax(q k^T scale) v) for a few query rows of ONE head.

    q_rows, dout_rows [R, d]; positions [R]; k, v [S, d] (natural token order); out_rows [R, d]
    (reading B5) or None.  Returns (dq [R, d], dk [S, d], dv [S, d]) in fp64.
    """
    q = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(dout_rows, dtype=np.float64)
    positions = np.asarray(positions, dtype=np.int64)
    R, d = q.shape
    S = k.shape[0]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    dq = np.zeros((R, d))
    dk = np.zeros((S, d))
    dv = np.zeros((S, d))
    block = max(1, (1 << 24) // S)               # rows per pass, only to bound memory
    key_pos = np.arange(S, dtype=np.int64)
    for r0 in range(0, R, block):
        r1 = min(R, r0 + block)
        s = (q[r0:r1] @ k.T) * scale                                  # [rows, S]
        if causal:
            s = np.where(key_pos[None, :] <= positions[r0:r1, None], s, -np.inf)
        mx = s.max(axis=1, keepdims=True)
        seen = np.isfinite(mx)
        e = np.exp(s - np.where(seen, mx, 0.0))
        den = e.sum(axis=1, keepdims=True)
        p = np.where(seen, e / np.where(den > 0, den, 1.0), 0.0)      # softmax rows (B4: all zero if nothing seen)
        out = p @ v if out_rows is None else np.asarray(out_rows, dtype=np.float64)[r0:r1]
        dp = do[r0:r1] @ v.T                                          # d loss / d p
        delta = (do[r0:r1] * out).sum(axis=1, keepdims=True)
        ds = p * (dp - delta)                                         # softmax Jacobian applied
        dq[r0:r1] = (ds @ k) * scale
        dk += (ds.T @ q[r0:r1]) * scale
        dv += p.T @ do[r0:r1]
    return dq, dk, dv


def stepwise_grads(q_rows, positions, k, v, dout_rows, n, rank, mask_mode, scale=None, looping=None):
    """The backward pass in the forward's arrival order (readings B1, B2), a few local rows of one head.

    Returns (dq [R, d], dk [S, d], dv [S, d], per_step) where per_step[s] = (tokens of step s,
    dq contribution of step s).
    """
    q = np.asarray(q_rows, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(dout_rows, dtype=np.float64)
    positions = np.asarray(positions, dtype=np.int64)
    R, d = q.shape
    S = k.shape[0]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    causal = mask_mode == sch.ZIGZAG_CAUSAL
    looping = sch.hamilton_rings(n) if looping is None else looping
    out, lse = att.dense_rows(q, positions, k, v, causal, scale)      # what the forward pass left behind
    delta = (do * out).sum(axis=1)
    dq = np.zeros((R, d))
    dk = np.zeros((S, d))
    dv = np.zeros((S, d))
    per_step = []
    for step in range(n):
        toks = np.asarray(att.step_tokens(n, rank, S, mask_mode, looping, step), dtype=np.int64)
        dq_s = np.zeros((R, d))
        for r in range(R):
            vis = toks[toks <= positions[r]] if causal else toks
            if vis.size == 0 or not np.isfinite(lse[r]):
                continue
            p = np.exp((k[vis] @ q[r]) * scale - lse[r])
            ds = p * (v[vis] @ do[r] - delta[r])
            dq_s[r] = (ds @ k[vis]) * scale
            dk[vis] += np.outer(ds, q[r]) * scale
            dv[vis] += np.outer(p, do[r])
        dq += dq_s
        per_step.append((toks, dq_s))
    return dq, dk, dv, per_step


def attention_bwd_flops(n, rank, S, mask_mode, Hq, d):
    """Five products of 2 d flops per visible (query, key) pair against the forward's two:
    q k^T, dout v^T, p^T dout, ds k, ds^T q."""
    return att.attention_flops(n, rank, S, mask_mode, Hq, d) * 5 // 2
