"""tasp_chunk_attn_static (the entry point that allocates nothing: workspace = a fixed array inside
the library) against tasp_chunk_attn on the same inputs, through the C ABI: two calls in a row, the
second on a smaller input, so that what the first call left in the shared array is under the second.

The file name sorts after every other test file on purpose."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2509_26541_amd import workloads as wl
from tests.helpers import max_abs, oracle_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2509_26541_amd import binding
    return binding


def _static_call(tb, w, q, k, v, sched, **kw):
    """Calls the entry point through the raw ABI into caller-owned out / lse."""
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:-1], float("nan"), dtype=torch.float32, device=q.device)
    a = tb._args(q, k, v, w.mask_mode, kw.get("order", tb.ORDER_TASP), kw.get("fuse_merge", False), 0.0,
                 kw.get("fuse_steps", False))
    a.out, a.lse = out.data_ptr(), lse.data_ptr()
    a.workspace, a.workspace_bytes = None, 0          # ignored by this entry point
    st = tb.lib.tasp_chunk_attn_static(sched.handle, C.byref(a), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == tb.OK, tb.strerror(st)
    return out, lse


CASES = [
    # first call (larger), second call (smaller); name, N, rank, S, Hq, Hkv, d, dtype, mask
    (("big_bf16", 8, 3, 8192, 8, 2, 128, "bf16", wl.ZIGZAG_CAUSAL), ("small_bf16", 8, 5, 8 * 2 * 100, 4, 2, 128, "bf16", wl.ZIGZAG_CAUSAL)),
    (("big_d64", 8, 1, 8 * 640, 4, 4, 64, "bf16", wl.FULL), ("small_fp32", 4, 2, 4 * 70, 2, 1, 64, "fp32", wl.FULL)),
]


@pytest.mark.parametrize("pair", CASES, ids=[c[0][0] for c in CASES])
@pytest.mark.parametrize("mode", [dict(fuse_merge=False), dict(fuse_merge=True), dict(fuse_steps=True)],
                         ids=["merge_kernel", "fused_merge", "one_launch"])
def test_static_scratch_matches_workspace_call(tb, pair, mode):
    for spec in pair:                                  # two calls in a row on the shared array
        name, n, rank, S, Hq, Hkv, d, dtype, mask = spec
        if mode.get("fuse_steps") and dtype != "bf16":
            continue
        w = wl.Workload(name, n, rank, S, Hq, Hkv, d, dtype, mask, seed=wl.BASE_SEED + 4242)
        q, k, v = wl.make_qkv(w)
        qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
        sched = tb.tasp_schedule(n, rank)
        print("static scratch: %s %s" % (name, mode), flush=True)
        ref_o, ref_l = tb.tasp_chunk_attn(qd, kd, vd, sched, mask, **mode)
        got_o, got_l = _static_call(tb, w, qd, kd, vd, sched, **mode)
        torch.cuda.synchronize()
        # the same kernels on the same inputs: identical bits
        assert torch.equal(got_l, ref_l)
        assert torch.equal(got_o, ref_o)
        # and both within the parity bar of the oracle
        tol_o, tol_l = (2e-2, 1e-3) if dtype == "bf16" else (1e-4, 1e-4)
        rows = list(range(0, w.L, 5))
        oo, ol = oracle_rows(w, q, k, v, rows)
        assert max_abs(got_o.float().cpu().numpy()[rows], oo) <= tol_o
        assert max_abs(got_l.cpu().numpy()[rows], ol) <= tol_l
        assert np.all(np.isfinite(got_l.cpu().numpy()))


def test_static_scratch_refuses_what_does_not_fit(tb):
    # bf16 running output of 32 Mi elements = 128 MiB > the 64 MiB array; only shapes are looked at
    # before the refusal, so small dummy buffers do
    n, S, Hq, d = 8, 8 * 32768, 8, 128
    sched = tb.tasp_schedule(n, 0)
    dummy = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    a = tb.AttnArgs()
    a.q = a.k = a.v = a.out = dummy.data_ptr()
    a.lse = dummy.data_ptr()
    a.S, a.Hq, a.Hkv, a.d, a.batch = S, Hq, Hq, d, 1
    a.dtype, a.mask_mode, a.order, a.fuse_merge = tb.DTYPE_BF16, tb.MASK_FULL, tb.ORDER_TASP, 1
    assert tb.lib.tasp_chunk_attn_workspace_bytes(sched.handle, C.byref(a)) > tb.STATIC_SCRATCH_BYTES
    st = tb.lib.tasp_chunk_attn_static(sched.handle, C.byref(a), None)
    assert st == tb.EWORKSPACE
    torch.cuda.synchronize()
