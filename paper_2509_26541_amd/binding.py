"""ctypes binding of libtasp.so: same names as include/tasp.h, argument marshalling only.

PyTorch supplies device memory and the HIP stream; every step of the path runs inside the library.
There is no fallback: if the library has not been built (python paper_2509_26541_amd/build.py, or
__graft_entry__.build()) importing this module raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtasp.so")

MASK_FULL, MASK_ZIGZAG_CAUSAL = 0, 1
DTYPE_FP32, DTYPE_BF16 = 0, 1
ORDER_TASP, ORDER_RING = 0, 1

OK, EINVAL, EUNSUPPORTED_N, EUNSUPPORTED_SHAPE, EALIGN, EWORKSPACE, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5, -6, -7

# every symbol include/tasp.h declares
EXPORTS = [
    "tasp_strerror", "tasp_schedule_create", "tasp_schedule_destroy", "tasp_schedule_n_ranks",
    "tasp_schedule_rank", "tasp_schedule_n_rings", "tasp_schedule_max_arc_load", "tasp_schedule_rings",
    "tasp_schedule_out_mapping", "tasp_schedule_in_mapping", "tasp_schedule_arrival", "tasp_subchunk_ranges",
    "tasp_step_segments", "tasp_chunk_attn_workspace_bytes", "tasp_chunk_attn", "tasp_step_attn",
    "tasp_lse_merge", "tasp_chunk_attn_flops", "tasp_chunk_attn_profile", "tasp_last_hip_error", "tasp_calibration_copy",
    "tasp_lse_merge_many", "tasp_calibration_mfma", "tasp_calibration_issue", "tasp_schedule_create_multinode",
    "tasp_chunk_attn_bwd_workspace_bytes", "tasp_chunk_attn_bwd", "tasp_chunk_attn_bwd_profile",
    "tasp_chunk_attn_bwd_flops", "tasp_chunk_attn_static",
]
STATIC_SCRATCH_BYTES = 64 << 20


class TaspError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        detail = " [HIP: %s]" % lib.tasp_last_hip_error().decode() if status == EHIP else ""
        super().__init__("%s: %s (status %d)%s" % (where, strerror(status), status, detail))


class AttnArgs(C.Structure):
    _fields_ = [
        ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("out", C.c_void_p), ("lse", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("S", C.c_int64),
        ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32), ("dtype", C.c_int32),
        ("mask_mode", C.c_int32), ("order", C.c_int32), ("fuse_merge", C.c_int32), ("softmax_scale", C.c_float),
        ("batch", C.c_int32), ("fuse_steps", C.c_int32),
    ]


class Profile(C.Structure):
    _fields_ = [("attn_ms", C.c_double), ("merge_ms", C.c_double), ("other_ms", C.c_double),
                ("attn_launches", C.c_int32), ("merge_launches", C.c_int32), ("other_launches", C.c_int32)]


class AttnBwdArgs(C.Structure):
    _fields_ = [
        ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("out", C.c_void_p), ("lse", C.c_void_p),
        ("dout", C.c_void_p), ("dq", C.c_void_p), ("dk", C.c_void_p), ("dv", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("S", C.c_int64),
        ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32), ("dtype", C.c_int32),
        ("mask_mode", C.c_int32), ("order", C.c_int32), ("softmax_scale", C.c_float), ("batch", C.c_int32),
        ("aux_stream", C.c_void_p), ("fuse_steps", C.c_int32),
    ]


class BwdProfile(C.Structure):
    _fields_ = [("dq_ms", C.c_double), ("dkv_ms", C.c_double), ("other_ms", C.c_double),
                ("dq_launches", C.c_int32), ("dkv_launches", C.c_int32), ("other_launches", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libtasp.so is not built: run `python paper_2509_26541_amd/build.py` "
                          "(there is no CPU fallback)")
    # PyTorch's ROCm wheel ships its own HIP runtime.  Importing torch first makes libtasp.so bind to
    # that same runtime; loaded the other way round the process ends up with two runtimes and the
    # library's launches fail with "no ROCm-capable device is detected".
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    p32 = C.POINTER(C.c_int32)
    lib.tasp_strerror.restype = C.c_char_p
    lib.tasp_strerror.argtypes = [C.c_int]
    lib.tasp_last_hip_error.restype = C.c_char_p
    lib.tasp_last_hip_error.argtypes = []
    lib.tasp_schedule_create.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
    lib.tasp_schedule_create_multinode.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
    lib.tasp_schedule_destroy.argtypes = [C.c_void_p]
    lib.tasp_schedule_destroy.restype = None
    for name in ("n_ranks", "rank", "n_rings", "max_arc_load"):
        f = getattr(lib, "tasp_schedule_" + name)
        f.argtypes = [C.c_void_p]
        f.restype = C.c_int32
    for name in ("rings", "out_mapping", "in_mapping", "arrival"):
        f = getattr(lib, "tasp_schedule_" + name)
        f.argtypes = [C.c_void_p]
        f.restype = p32
    lib.tasp_subchunk_ranges.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                         C.POINTER(C.c_int64), p32]
    lib.tasp_step_segments.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.POINTER(C.c_int64), p32, C.c_int32, p32]
    lib.tasp_chunk_attn_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(AttnArgs)]
    lib.tasp_chunk_attn_workspace_bytes.restype = C.c_size_t
    lib.tasp_chunk_attn.argtypes = [C.c_void_p, C.POINTER(AttnArgs), C.c_void_p]
    lib.tasp_chunk_attn_static.argtypes = [C.c_void_p, C.POINTER(AttnArgs), C.c_void_p]
    lib.tasp_chunk_attn_profile.argtypes = [C.c_void_p, C.POINTER(AttnArgs), C.c_void_p, C.POINTER(Profile)]
    lib.tasp_step_attn.argtypes = [C.c_void_p, C.POINTER(AttnArgs), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.tasp_lse_merge.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                   C.c_int32, C.c_void_p]
    lib.tasp_calibration_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.tasp_lse_merge_many.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32,
                                        C.c_int64, C.c_int32, C.c_int32, C.c_void_p]
    lib.tasp_calibration_mfma.argtypes = [C.c_int32, C.POINTER(C.c_double), C.c_void_p]
    lib.tasp_calibration_issue.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.tasp_chunk_attn_flops.argtypes = [C.c_void_p, C.POINTER(AttnArgs)]
    lib.tasp_chunk_attn_flops.restype = C.c_double
    lib.tasp_chunk_attn_bwd_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(AttnBwdArgs)]
    lib.tasp_chunk_attn_bwd_workspace_bytes.restype = C.c_size_t
    lib.tasp_chunk_attn_bwd.argtypes = [C.c_void_p, C.POINTER(AttnBwdArgs), C.c_void_p]
    lib.tasp_chunk_attn_bwd_profile.argtypes = [C.c_void_p, C.POINTER(AttnBwdArgs), C.c_void_p, C.POINTER(BwdProfile)]
    lib.tasp_chunk_attn_bwd_flops.argtypes = [C.c_void_p, C.POINTER(AttnBwdArgs)]
    lib.tasp_chunk_attn_bwd_flops.restype = C.c_double
    return lib


lib = _load()


def strerror(status):
    return lib.tasp_strerror(int(status)).decode()


def _check(status, where):
    if status != OK:
        raise TaspError(status, where)


class Schedule:
    """tasp_schedule(N, rank): owns a tasp_schedule_t; arrays are copied out as numpy int32."""

    def __init__(self, n_ranks, rank, ranks_per_node=None):
        self._h = C.c_void_p()
        if ranks_per_node is None:
            _check(lib.tasp_schedule_create(n_ranks, rank, C.byref(self._h)), "tasp_schedule_create")
        else:
            if ranks_per_node <= 0 or n_ranks % ranks_per_node:
                raise ValueError("n_ranks must be a multiple of ranks_per_node")
            _check(lib.tasp_schedule_create_multinode(ranks_per_node, n_ranks // ranks_per_node, rank, C.byref(self._h)),
                   "tasp_schedule_create_multinode")
        n = lib.tasp_schedule_n_ranks(self._h)
        m = lib.tasp_schedule_n_rings(self._h)
        self.n_ranks, self.rank, self.n_rings = n, lib.tasp_schedule_rank(self._h), m
        self.max_arc_load = lib.tasp_schedule_max_arc_load(self._h)
        self.rings = np.ctypeslib.as_array(lib.tasp_schedule_rings(self._h), (m, n)).copy()
        self.out_mapping = np.ctypeslib.as_array(lib.tasp_schedule_out_mapping(self._h), (n, n)).copy()
        self.in_mapping = np.ctypeslib.as_array(lib.tasp_schedule_in_mapping(self._h), (n, n)).copy()
        self.arrival = np.ctypeslib.as_array(lib.tasp_schedule_arrival(self._h), (n, m)).copy()

    @property
    def handle(self):
        return self._h

    def subchunk_ranges(self, S, mask_mode, ring, src_rank):
        r = (C.c_int64 * 4)()
        cnt = C.c_int32()
        _check(lib.tasp_subchunk_ranges(self._h, S, mask_mode, ring, src_rank, r, C.byref(cnt)),
               "tasp_subchunk_ranges")
        return [(r[2 * i], r[2 * i + 1]) for i in range(cnt.value)]

    def step_segments(self, S, mask_mode, step, q_block, order=ORDER_TASP, cap=256):
        seg = (C.c_int64 * (2 * cap))()
        diag = (C.c_int32 * cap)()
        cnt = C.c_int32()
        _check(lib.tasp_step_segments(self._h, S, mask_mode, order, step, q_block, seg, diag, cap, C.byref(cnt)),
               "tasp_step_segments")
        return [(seg[2 * i], seg[2 * i + 1], diag[i]) for i in range(cnt.value)]

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:            # module globals may already be gone at interpreter exit
            lib.tasp_schedule_destroy(h)


def tasp_schedule(n_ranks, rank):
    return Schedule(n_ranks, rank)


def tasp_schedule_multinode(ranks_per_node, n_nodes, rank):
    """The (m-K_m-m)^u scheme: m = ranks_per_node rings over m * n_nodes ranks."""
    return Schedule(ranks_per_node * n_nodes, rank, ranks_per_node=ranks_per_node)


def _torch():
    import torch
    return torch


def _args(q, k, v, mask_mode, order, fuse_merge, softmax_scale, fuse_steps=False):
    torch = _torch()
    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise ValueError("q, k, v must be device tensors")
    if not (q.is_contiguous() and k.is_contiguous() and v.is_contiguous()):
        raise ValueError("q, k, v must be contiguous")
    if q.dtype != k.dtype or q.dtype != v.dtype or q.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("q, k, v must share dtype float32 or bfloat16")
    if q.dim() not in (3, 4) or k.dim() != q.dim() or v.shape != k.shape or q.shape[-1] != k.shape[-1]:
        raise ValueError("expected q [L, Hq, d] and k, v [S, Hkv, d], or all three with a leading batch dimension")
    if q.dim() == 4 and q.shape[0] != k.shape[0]:
        raise ValueError("q and k, v must hold the same number of sequences")
    a = AttnArgs()
    a.q, a.k, a.v = q.data_ptr(), k.data_ptr(), v.data_ptr()
    a.S, a.Hq, a.Hkv, a.d = k.shape[-3], q.shape[-2], k.shape[-2], q.shape[-1]
    a.batch = q.shape[0] if q.dim() == 4 else 1
    a.dtype = DTYPE_FP32 if q.dtype == torch.float32 else DTYPE_BF16
    a.mask_mode, a.order, a.fuse_merge, a.softmax_scale = mask_mode, order, int(bool(fuse_merge)), softmax_scale
    a.fuse_steps = int(bool(fuse_steps))
    return a


class ChunkAttnPlan:
    """Buffers of one tasp_chunk_attn shape (out, lse, workspace), so that repeated calls allocate nothing."""

    def __init__(self, schedule, q, k, v, mask_mode, order=ORDER_TASP, fuse_merge=False, softmax_scale=0.0,
                 fuse_steps=False):
        torch = _torch()
        self.schedule = schedule
        self.args = _args(q, k, v, mask_mode, order, fuse_merge, softmax_scale, fuse_steps)
        if q.shape[-3] * schedule.n_ranks != k.shape[-3]:
            raise ValueError("q must hold S / N local rows")
        self.out = torch.empty_like(q)
        self.lse = torch.empty(q.shape[:-1], dtype=torch.float32, device=q.device)
        nbytes = lib.tasp_chunk_attn_workspace_bytes(schedule.handle, C.byref(self.args))
        self.workspace = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=q.device)
        self.args.out, self.args.lse = self.out.data_ptr(), self.lse.data_ptr()
        self.args.workspace, self.args.workspace_bytes = self.workspace.data_ptr(), nbytes
        self._keep = (q, k, v)

    def run(self, stream=None):
        torch = _torch()
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        _check(lib.tasp_chunk_attn(self.schedule.handle, C.byref(self.args), C.c_void_p(s)), "tasp_chunk_attn")
        return self.out, self.lse

    def profile(self, stream=None):
        """Runs the call once with per-launch HIP-event timing; returns a Profile (milliseconds)."""
        torch = _torch()
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        prof = Profile()
        _check(lib.tasp_chunk_attn_profile(self.schedule.handle, C.byref(self.args), C.c_void_p(s), C.byref(prof)),
               "tasp_chunk_attn_profile")
        return prof

    def flops(self):
        return lib.tasp_chunk_attn_flops(self.schedule.handle, C.byref(self.args))


def tasp_chunk_attn(q, k, v, schedule, mask_mode, order=ORDER_TASP, fuse_merge=False, softmax_scale=0.0,
                    fuse_steps=False):
    """One rank's forward pass (Algorithm 3).  Returns (out [L, Hq, d] in q's dtype, lse [L, Hq] fp32)."""
    return ChunkAttnPlan(schedule, q, k, v, mask_mode, order, fuse_merge, softmax_scale, fuse_steps).run()


class ChunkAttnBwdPlan:
    """Buffers of one tasp_chunk_attn_bwd shape (dq, dk, dv, workspace), so that repeated calls allocate nothing."""

    def __init__(self, schedule, q, k, v, out, lse, dout, mask_mode, order=ORDER_TASP, softmax_scale=0.0,
                 aux_stream=None, fuse_steps=False):
        """aux_stream: a torch.cuda.Stream for the dk/dv kernels (None: everything on one stream)."""
        torch = _torch()
        fa = _args(q, k, v, mask_mode, order, True, softmax_scale)
        if q.shape[-3] * schedule.n_ranks != k.shape[-3]:
            raise ValueError("q must hold S / N local rows")
        for name, t, like in (("out", out, q), ("dout", dout, q)):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == like.dtype and t.shape == like.shape):
                raise ValueError("%s must be a contiguous device tensor shaped and typed like q" % name)
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and lse.shape == q.shape[:-1]):
            raise ValueError("lse must be a contiguous fp32 device tensor [.., L, Hq]")
        self.schedule = schedule
        a = AttnBwdArgs()
        a.q, a.k, a.v, a.out, a.lse, a.dout = (t.data_ptr() for t in (q, k, v, out, lse, dout))
        a.S, a.Hq, a.Hkv, a.d, a.batch, a.dtype = fa.S, fa.Hq, fa.Hkv, fa.d, fa.batch, fa.dtype
        a.mask_mode, a.order, a.softmax_scale = mask_mode, order, softmax_scale
        a.fuse_steps = int(bool(fuse_steps))
        self.dq, self.dk, self.dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        a.dq, a.dk, a.dv = self.dq.data_ptr(), self.dk.data_ptr(), self.dv.data_ptr()
        nbytes = lib.tasp_chunk_attn_bwd_workspace_bytes(schedule.handle, C.byref(a))
        self.workspace = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=q.device)
        a.workspace, a.workspace_bytes = self.workspace.data_ptr(), nbytes
        a.aux_stream = aux_stream.cuda_stream if aux_stream is not None else None
        self.args = a
        self._keep = (q, k, v, out, lse, dout, aux_stream)

    def run(self, stream=None):
        torch = _torch()
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        _check(lib.tasp_chunk_attn_bwd(self.schedule.handle, C.byref(self.args), C.c_void_p(s)), "tasp_chunk_attn_bwd")
        return self.dq, self.dk, self.dv

    def profile(self, stream=None):
        torch = _torch()
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        prof = BwdProfile()
        _check(lib.tasp_chunk_attn_bwd_profile(self.schedule.handle, C.byref(self.args), C.c_void_p(s), C.byref(prof)),
               "tasp_chunk_attn_bwd_profile")
        return prof

    def flops(self):
        return lib.tasp_chunk_attn_bwd_flops(self.schedule.handle, C.byref(self.args))


def tasp_chunk_attn_static(q, k, v, out, lse, schedule, mask_mode, order=ORDER_TASP, fuse_merge=False,
                           softmax_scale=0.0, fuse_steps=False):
    """tasp_chunk_attn into the caller's out / lse with the library's own fixed scratch as workspace:
    nothing is allocated, here or in the library.  Raises TaspError(EWORKSPACE) beyond STATIC_SCRATCH_BYTES."""
    torch = _torch()
    a = _args(q, k, v, mask_mode, order, fuse_merge, softmax_scale, fuse_steps)
    if not (out.is_cuda and out.is_contiguous() and out.dtype == q.dtype and out.shape == q.shape):
        raise ValueError("out must be a contiguous device tensor shaped and typed like q")
    if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and lse.shape == q.shape[:-1]):
        raise ValueError("lse must be a contiguous fp32 device tensor [.., L, Hq]")
    a.out, a.lse = out.data_ptr(), lse.data_ptr()
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_chunk_attn_static(schedule.handle, C.byref(a), C.c_void_p(s)), "tasp_chunk_attn_static")
    return out, lse


def tasp_chunk_attn_bwd(q, k, v, out, lse, dout, schedule, mask_mode, order=ORDER_TASP, softmax_scale=0.0,
                        aux_stream=None, fuse_steps=False):
    """One rank's backward pass in the forward's arrival order.  out, lse: what tasp_chunk_attn returned
    for the same inputs.  Returns (dq like q, dk like k, dv like v); dk, dv are this rank's contribution."""
    return ChunkAttnBwdPlan(schedule, q, k, v, out, lse, dout, mask_mode, order, softmax_scale, aux_stream,
                            fuse_steps).run()


def tasp_step_attn(q, k, v, schedule, mask_mode, step, order=ORDER_TASP, softmax_scale=0.0):
    """Partial (out_s fp32, lse_s fp32) of one step, before any merge."""
    torch = _torch()
    a = _args(q, k, v, mask_mode, order, False, softmax_scale)
    o = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    lse = torch.empty(q.shape[:-1], dtype=torch.float32, device=q.device)
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_step_attn(schedule.handle, C.byref(a), step, o.data_ptr(), lse.data_ptr(), C.c_void_p(s)),
           "tasp_step_attn")
    return o, lse


def tasp_calibration_copy(dst, src):
    """Streams src into dst (same-size contiguous device tensors) with the library's copy kernel."""
    torch = _torch()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise ValueError("device tensors of equal byte size expected")
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, C.c_void_p(s)), "tasp_calibration_copy")
    return dst


def tasp_calibration_mfma(iters):
    """Launches the matrix-pipe calibration kernel on the current stream; returns its flop count."""
    torch = _torch()
    flops = C.c_double(0.0)
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_calibration_mfma(int(iters), C.byref(flops), C.c_void_p(s)), "tasp_calibration_mfma")
    return flops.value


def tasp_calibration_issue(kind, per_slot, iters=2000):
    """Shader-clock cycles per slot of the issue-cost calibration (kind 0: per_slot fma, 1: per_slot
    exp, 2: eight fma + per_slot ds_read_b128, each behind one matrix instruction): the slowest
    wavefront of each of the 256 workgroups, averaged over the workgroups."""
    torch = _torch()
    out = torch.zeros((256, 8), dtype=torch.int64, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_calibration_issue(int(kind), int(per_slot), int(iters), out.data_ptr(), C.c_void_p(s)),
           "tasp_calibration_issue")
    torch.cuda.synchronize()
    return float(out.max(dim=1).values.double().mean()) / 16.0


def tasp_lse_merge_many(o_parts, lse_parts, o_out=None, lse_out=None):
    """All partial pairs merged in one pass.  o_parts: list of fp32 device tensors [rows, heads, d],
    lse_parts: list of [rows, heads]; returns (o_out, lse_out) (allocated if not given)."""
    torch = _torch()
    n = len(o_parts)
    if n == 0 or n != len(lse_parts):
        raise ValueError("equally many out and lse partials, at least one")
    for t in list(o_parts) + list(lse_parts):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
            raise ValueError("contiguous fp32 device tensors expected")
    rows, heads, d = o_parts[0].shape
    for o, l in zip(o_parts, lse_parts):
        if tuple(o.shape) != (rows, heads, d) or tuple(l.shape) != (rows, heads):
            raise ValueError("all partials must have the same shape")
    if o_out is None:
        o_out = torch.empty_like(o_parts[0])
    if lse_out is None:
        lse_out = torch.empty_like(lse_parts[0])
    op = (C.c_void_p * n)(*[t.data_ptr() for t in o_parts])
    lp = (C.c_void_p * n)(*[t.data_ptr() for t in lse_parts])
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_lse_merge_many(o_out.data_ptr(), lse_out.data_ptr(), op, lp, n, rows, heads, d, C.c_void_p(s)),
           "tasp_lse_merge_many")
    return o_out, lse_out


def tasp_lse_merge(o_acc, lse_acc, o_part, lse_part):
    """update_out_lse in place on (o_acc, lse_acc); all fp32 device tensors [rows, heads, d] / [rows, heads]."""
    torch = _torch()
    for t in (o_acc, lse_acc, o_part, lse_part):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32):
            raise ValueError("fp32 contiguous device tensors expected")
    rows, heads, d = o_acc.shape
    if o_part.shape != o_acc.shape or lse_acc.shape != (rows, heads) or lse_part.shape != (rows, heads):
        raise ValueError("shape mismatch")
    s = torch.cuda.current_stream().cuda_stream
    _check(lib.tasp_lse_merge(o_acc.data_ptr(), lse_acc.data_ptr(), o_part.data_ptr(), lse_part.data_ptr(),
                              rows, heads, d, C.c_void_p(s)), "tasp_lse_merge")
    return o_acc, lse_acc
