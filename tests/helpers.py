"""Shared by the GPU parity tests: evaluates the oracle on chosen local rows of a workload."""
import numpy as np

from oracle import attention as att
from oracle import schedule as sch


def oracle_rows(w, q, k, v, rows, heads=None):
    """Dense fp64 attention (oracle) for local rows `rows` and query heads `heads` of workload w.
    q, k, v are the CPU tensors handed to the GPU (bf16 -> fp64 is exact).
    Returns (out [len(rows), len(heads), d], lse [len(rows), len(heads)])."""
    heads = list(range(w.Hq)) if heads is None else list(heads)
    rows = list(rows)
    pos = np.asarray(sch.local_positions(w.n_ranks, w.rank, w.S, w.mask_mode), dtype=np.int64)[rows]
    causal = w.mask_mode == sch.ZIGZAG_CAUSAL
    out = np.zeros((len(rows), len(heads), w.d))
    lse = np.zeros((len(rows), len(heads)))
    by_group = {}
    for j, h in enumerate(heads):
        by_group.setdefault(h * w.Hkv // w.Hq, []).append((j, h))
    for g, members in by_group.items():
        kg = k[:, g].double().numpy()
        vg = v[:, g].double().numpy()
        for j, h in members:
            qh = q[rows, h].double().numpy()
            out[:, j], lse[:, j] = att.dense_rows(qh, pos, kg, vg, causal)
    return out, lse


def oracle_grads(w, q, k, v, dout, rows=None, out=None, progress=None):
    """Dense fp64 gradients (oracle) of sum(dout * out) for workload w, all heads; `rows` restricts the
    local query rows that take part (the gradient is linear in dout, so this equals zeroing dout
    elsewhere); `out` [L, Hq, d] is the stored forward output delta is taken from (None: the exact
    one).  Returns (dq [len(rows), Hq, d], dk [S, Hkv, d], dv [S, Hkv, d])."""
    from oracle import attention_bwd as bwd
    rows = list(range(w.L)) if rows is None else list(rows)
    pos = np.asarray(sch.local_positions(w.n_ranks, w.rank, w.S, w.mask_mode), dtype=np.int64)[rows]
    causal = w.mask_mode == sch.ZIGZAG_CAUSAL
    dq = np.zeros((len(rows), w.Hq, w.d))
    dk = np.zeros((w.S, w.Hkv, w.d))
    dv = np.zeros((w.S, w.Hkv, w.d))
    for h in range(w.Hq):
        g = h * w.Hkv // w.Hq
        a, b, c = bwd.dense_grads(q[rows, h].double().numpy(), pos, k[:, g].double().numpy(), v[:, g].double().numpy(),
                                  dout[rows, h].double().numpy(), causal,
                                  out_rows=None if out is None else out[rows, h].double().numpy())
        dq[:, h] = a
        dk[:, g] += b
        dv[:, g] += c
        if progress is not None and (h + 1) % 8 == 0:
            progress("oracle: %d of %d heads" % (h + 1, w.Hq))
    return dq, dk, dv


def max_abs(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    both_ninf = np.isneginf(a) & np.isneginf(b)
    diff = np.where(both_ninf, 0.0, np.abs(a - b))
    return float(np.max(diff)) if diff.size else 0.0
