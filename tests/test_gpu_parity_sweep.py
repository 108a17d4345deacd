"""Seeded sweep over valid small shapes: forward and backward of the HIP path against the fp64 oracle.

The hand-picked cases of the other parity tests sit at known edges; this one draws the combination
(number of ranks, rank, sequence length, heads, head dimension, dtype, mask, order, batch, the two
fuse modes, second stream, multi-node schedule) at random from a fixed seed, every element checked,
to the same bars: forward max-abs 2e-2 / 1e-3 (bf16) and 1e-4 (fp32); backward
|err| <= 2^-7 |ref| + 2^-8 max|ref| (bf16) and 1e-4 max(1, max|ref|) (fp32).  The backward call gets
the out and lse the forward call stored, and the oracle takes delta from that same stored out."""
import numpy as np
import pytest
import torch

from paper_2509_26541_amd import workloads as wl
from tests.helpers import max_abs, oracle_grads, oracle_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2509_26541_amd import binding
    return binding


def draw(rng, tb, index, seed):
    n = int(rng.choice([4, 8, 8, 8, 12, 16, 20]))
    multinode = n in (8, 16) and rng.random() < 0.2
    rank = int(rng.integers(0, n))
    mode = wl.ZIGZAG_CAUSAL if rng.random() < 0.65 else wl.FULL
    unit = 2 * n if mode == wl.ZIGZAG_CAUSAL else n
    S = unit * int(rng.choice([1, 2, 3, 7, 16, 33, 64, 100, 129, 200, 257]))
    if S > 9000:
        S = unit * 33
    Hkv, G, d = int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 4])), int(rng.choice([64, 128]))
    dtype = "bf16" if rng.random() < 0.8 else "fp32"
    base = wl.CONFIGS[int(rng.choice([1, 2]))]
    w = wl.Workload("sweep_%d_%d" % (seed, index), n, rank, S, Hkv * G, Hkv, d, dtype, mode, k_scale=base.k_scale,
                    seed=wl.BASE_SEED + 5000 + 1000 * seed + 13 * index)
    opts = dict(order=tb.ORDER_RING if rng.random() < 0.25 else tb.ORDER_TASP, batch=int(rng.choice([1, 1, 2, 3])),
                fuse_steps=bool(dtype == "bf16" and rng.random() < 0.35), fuse_merge=bool(rng.random() < 0.6),
                aux=bool(rng.random() < 0.3), multinode=multinode)
    return w, opts


@pytest.mark.parametrize("seed", [1, 2])
def test_random_valid_shapes(tb, seed):
    rng = np.random.default_rng(seed)
    for index in range(30):
        w, o = draw(rng, tb, index, seed)
        tag = "%s: n=%d rank=%d S=%d Hq=%d Hkv=%d d=%d %s mask=%d %s" % (w.name, w.n_ranks, w.rank, w.S, w.Hq, w.Hkv, w.d,
                                                                      w.dtype, w.mask_mode, o)
        print(tag, flush=True)
        sched = (tb.tasp_schedule_multinode(w.n_ranks // 2, 2, w.rank) if o["multinode"]
                 else tb.tasp_schedule(w.n_ranks, w.rank))
        B = o["batch"]
        seqs = []
        for b in range(B):
            wb = wl.Workload(w.name, w.n_ranks, w.rank, w.S, w.Hq, w.Hkv, w.d, w.dtype, w.mask_mode, k_scale=w.k_scale,
                             seed=w.seed + 1000003 * b)
            seqs.append(wl.make_qkv(wb) + (wl.make_dout(wb),))
        q, k, v, do = (torch.stack([s[i] for s in seqs]) if B > 1 else seqs[0][i] for i in range(4))
        qd, kd, vd, dod = q.cuda(), k.cuda(), v.cuda(), do.cuda()
        out, lse = tb.tasp_chunk_attn(qd, kd, vd, sched, w.mask_mode, order=o["order"], fuse_merge=o["fuse_merge"],
                                      fuse_steps=o["fuse_steps"])
        side = torch.cuda.Stream() if o["aux"] else None
        dq, dk, dv = tb.tasp_chunk_attn_bwd(qd, kd, vd, out, lse, dod, sched, w.mask_mode, order=o["order"],
                                            aux_stream=side, fuse_steps=o["fuse_steps"])
        torch.cuda.synchronize()
        tol_o, tol_l = (2e-2, 1e-3) if w.dtype == "bf16" else (1e-4, 1e-4)
        for b in range(B):
            qb, kb, vb, dob = seqs[b]
            pick = (lambda t: t[b]) if B > 1 else (lambda t: t)
            ro, rl = oracle_rows(w, qb, kb, vb, range(w.L))
            lb = pick(lse).cpu().numpy()
            assert np.all(np.isfinite(lb)), tag
            eo, el = max_abs(pick(out).float().cpu().numpy(), ro), max_abs(lb, rl)
            assert eo <= tol_o and el <= tol_l, "%s seq %d: out err %.3e, lse err %.3e" % (tag, b, eo, el)
            rq, rk, rv = oracle_grads(w, qb, kb, vb, dob, out=pick(out).cpu())
            for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
                g = pick(got).float().cpu().numpy().astype(np.float64)
                assert np.all(np.isfinite(g)), (tag, name)
                if w.dtype == "bf16":
                    bound = np.abs(ref) / 128 + np.abs(ref).max() / 256 + 1e-30
                    worst = float((np.abs(g - ref) / bound).max())
                else:
                    worst = float(np.abs(g - ref).max() / (1e-4 * max(1.0, np.abs(ref).max())))
                assert worst <= 1.0, "%s seq %d %s: %.3f of the bound" % (tag, b, name, worst)
