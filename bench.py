"""Benchmark of one rank's TASP-ordered chunked attention on one MI355X.

A "step" is one whole tasp_chunk_attn call (all N steps of Algorithm 3: step attention over the
arriving sub-chunks, update_out_lse, final cast) over one batch of seeded synthetic input that is
already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--fuse-merge 1|0]

The timed call folds update_out_lse into the attention epilogue (fuse_merge, the faster of the two
modes of the library); the same call with the separate HBM-bound merge kernel is timed next to it
("other_merge_mode") and provides the merge kernel's GB/s ("merge").  `value` comes from the wall
clock around the K timed calls (synchronised on both sides); "ms_per_step_median_events" is the
median of the K calls timed one by one with HIP events on the launch stream.  With the default
workload the line also carries "other_workloads": the same call on the 256K, 512K and 1M workloads
(device-generated inputs of the same shapes and distributions, at most three timed calls each).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3        # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0
N_SIMD, CLOCK_HZ = 256 * 4, 2.4e9

# The second bound of the bf16 attention kernel: the vector issue port of a SIMD.  Measured on this
# chip with issue microbenchmarks: a matrix instruction occupies the port for 12 cycles, a plain
# vector instruction for 4, an exponential for 8, and a KiB of LDS data returned to registers for 4.
# Per 64-key tile and wavefront (32 queries) the kernel issues, on its common path, the counts below
# (from the generated code); flops of that unit of work divided by its port cycles, times the chip's
# SIMDs and the nominal clock, is the rate at which the port alone would let the kernel run.
PORT_CYCLES = {"mfma": 12, "valu": 4, "exp": 8, "lds_kib": 4}
TILE_MIX = {128: {"mfma": 32, "valu": 107, "exp": 33, "lds_kib": 32},
            64: {"mfma": 16, "valu": 105, "exp": 33, "lds_kib": 16}}


def valu_peak_tflops(d):
    mix = TILE_MIX[d]
    cycles = sum(PORT_CYCLES[k] * n for k, n in mix.items())
    return 4.0 * d * 32 * 64 / cycles * N_SIMD * CLOCK_HZ / 1e12


def measure_port_cycles(tb):
    """The port-cycle figures above, measured on this GPU (tasp_calibration_issue): a slot of one
    matrix instruction and n instructions of a kind, issued by two wavefronts per SIMD, lasts
    2 x (matrix + n x kind) port cycles once the port bounds it; two values of n give both terms."""
    f8, f12 = tb.tasp_calibration_issue(0, 8), tb.tasp_calibration_issue(0, 12)
    e4, e8 = tb.tasp_calibration_issue(1, 4), tb.tasp_calibration_issue(1, 8)
    l1, l2 = tb.tasp_calibration_issue(2, 1), tb.tasp_calibration_issue(2, 2)
    valu = (f12 - f8) / 8.0
    return {"valu": valu, "mfma": f8 / 2.0 - 8.0 * valu, "exp": (e8 - e4) / 8.0, "lds_kib": (l2 - l1) / 2.0,
            "cycles_per_slot": {"fma8": f8, "fma12": f12, "exp4": e4, "exp8": e8, "fma8_lds1": l1, "fma8_lds2": l2}}


def cpu_baseline(w, q, k, v, budget_s=12.0):
    """The oracle, as it stands, on a bounded sample of the same workload: dense fp64 attention of
    sampled local rows for all heads of one KV group, sized by a short calibration to ~budget_s."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import attention as att
    from oracle import schedule as sch
    from paper_2509_26541_amd import workloads as wl
    from tests.helpers import oracle_rows

    G = w.Hq // w.Hkv
    heads = list(range(G))                       # the query heads of KV head 0
    pos = np.asarray(sch.local_positions(w.n_ranks, w.rank, w.S, w.mask_mode), dtype=np.int64)
    causal = w.mask_mode == sch.ZIGZAG_CAUSAL

    def run(rows):
        t0 = time.perf_counter()
        oracle_rows(w, q, k, v, rows, heads)
        dt = time.perf_counter() - t0
        pairs = float(np.sum(pos[rows] + 1)) if causal else float(len(rows)) * w.S
        return dt, 4.0 * w.d * len(heads) * pairs

    all_rows = wl.sample_rows(w, 16384)
    # two probes separate the fixed cost (casting one KV head to fp64) from the cost per row
    p8 = all_rows[:: max(1, len(all_rows) // 8)][:8]
    p64 = all_rows[:: max(1, len(all_rows) // 64)][:64]
    t8, _ = run(p8)
    t64, _ = run(p64)
    per_row = max((t64 - t8) / max(len(p64) - len(p8), 1), 1e-6)
    fixed = max(t8 - per_row * len(p8), 0.0)
    n = int(max(8, min(len(all_rows), (budget_s - fixed) / per_row)))
    rows = all_rows[:: max(1, len(all_rows) // n)][:n]
    dt, flops = run(rows)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "sample": "%d sampled local rows x %d query heads (KV head 0), dense fp64 over all %d keys, %.1f s; "
                  "host has %d cores" % (len(rows), len(heads), w.S, dt, len(os.sched_getaffinity(0))),
    }


def device_qkv(w, torch, dev):
    """Inputs of workload w drawn on the device: same shapes, dtypes and value recipe as
    workloads.make_qkv (N(0,1); K scaled; a seeded 1 % of the key rows scaled for the outlier workload),
    from a seeded device generator instead of the CPU one, which takes minutes at a million tokens."""
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    draw = lambda shape: torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16 if w.dtype == "bf16" else torch.float32)
    qd, kd, vd = draw((w.L, w.Hq, w.d)), draw((w.S, w.Hkv, w.d)), draw((w.S, w.Hkv, w.d))
    if w.k_scale != 1.0:
        kd *= w.k_scale
    if w.outlier_frac > 0.0:
        rows = torch.randperm(w.S, generator=g, device=dev)[: int(w.outlier_frac * w.S)]
        kd[rows] *= w.outlier_scale
    return qd, kd, vd


def other_workloads(tb, wl, torch, dev, order, args, t_start, cap_s=150.0):
    """The forward call on the three larger workloads (256K, 512K, 1M): value and the attention
    launch's fraction of the bf16 peak.  Inputs are drawn on the device (device_qkv).  At most three
    timed calls each, and none is started once the bench has run for cap_s seconds."""
    out = []
    for idx in (2, 3, 4):
        w = wl.CONFIGS[idx]
        if time.perf_counter() - t_start > cap_s:
            out.append({"workload": w.name, "skipped": "wall-clock cap of the bench reached"})
            continue
        qd, kd, vd = device_qkv(w, torch, dev)
        sched = tb.tasp_schedule_multinode(w.n_ranks // args.nodes, args.nodes, w.rank) if args.nodes > 1 else tb.tasp_schedule(w.n_ranks, w.rank)
        plan = tb.ChunkAttnPlan(sched, qd, kd, vd, w.mask_mode, order=order, fuse_merge=True)
        flops = plan.flops()
        plan.run()
        torch.cuda.synchronize()
        steps = min(3, args.steps)
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.run()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        pr = plan.profile()
        launch = flops / (pr.attn_ms * 1e-3) / 1e12
        out.append({"workload": w.name, "S": w.S, "L": w.L, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d, "steps": steps,
                    "ms_per_step": ms, "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
                    "roofline": {"bound": "mfma", "kernel": "attn_bf16_kernel", "achieved": launch, "peak": PEAK_BF16_TFLOPS,
                                 "frac": launch / PEAK_BF16_TFLOPS, "avg_launch_ms": pr.attn_ms / max(pr.attn_launches, 1),
                                 "launches_per_call": pr.attn_launches}})
        del plan, qd, kd, vd
        torch.cuda.empty_cache()
    return out


def main():
    t_start = time.perf_counter()
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="1..5, the workload list of BASELINE.json")
    ap.add_argument("--fuse-merge", type=int, default=1)
    ap.add_argument("--fuse-steps", type=int, default=0,
                    help="1: time the form with all steps in one launch as the main leg (bf16; the default line "
                         "reports it as `single_launch` beside the step-by-step `value`)")
    ap.add_argument("--order", choices=["tasp", "ring"], default="tasp")
    ap.add_argument("--nodes", type=int, default=0,
                    help="U > 1: the (m-K_m-m)^U ring scheme for U nodes of N/U ranks (m rings) instead of the N-1 rings of K_N")
    ap.add_argument("--batch", type=int, default=1,
                    help="B > 1: B sequences of the workload's shape in one call (sequence b seeded with seed + 1000 b)")
    ap.add_argument("--grid", default="",
                    help="HEADS,SEQ: a shape of the paper's own grid (Sec. 5.1.2: MHA, d = 64, bf16) on 8 ranks "
                         "instead of --config; combine with --batch")
    ap.add_argument("--no-backward", action="store_true", help="skip the leg that times the backward pass (bf16 workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-mode", action="store_true",
                    help="skip the legs that run the other merge mode, the single launch and the backward pass on "
                         "two streams (profiler runs: one kind of launch per kernel)")
    ap.add_argument("--device-inputs", action="store_true",
                    help="draw the inputs on the device (same recipe, another generator): the 1M workload in seconds")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB copy with the library's copy kernel (scales profiler traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one rank's share on ONE GPU; --gpus N > 1 is not part of this build "
              "(no collectives, no sharding).", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2509_26541_amd import binding as tb
    from paper_2509_26541_amd import workloads as wl

    if args.grid:
        heads, seq = (int(x) for x in args.grid.split(","))
        w = wl.paper_grid(heads, seq)
    else:
        w = wl.CONFIGS[args.config - 1]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.device_inputs:
        qd, kd, vd = device_qkv(w, torch, dev)
        q, k, v = (None, None, None) if args.no_cpu_baseline else (qd.cpu(), kd.cpu(), vd.cpu())
    else:
        q, k, v = wl.make_qkv(w)
        qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    if args.batch > 1:
        import dataclasses
        more = [wl.make_qkv(dataclasses.replace(w, seed=w.seed + 1000 * b)) for b in range(1, args.batch)]
        qd, kd, vd = (torch.stack([x] + [m[i].to(dev) for m in more]) for i, x in enumerate((qd, kd, vd)))
        del more
    if args.nodes > 1:
        sched = tb.tasp_schedule_multinode(w.n_ranks // args.nodes, args.nodes, w.rank)
    else:
        sched = tb.tasp_schedule(w.n_ranks, w.rank)
    order = tb.ORDER_TASP if args.order == "tasp" else tb.ORDER_RING
    plan = tb.ChunkAttnPlan(sched, qd, kd, vd, w.mask_mode, order=order, fuse_merge=bool(args.fuse_merge),
                            fuse_steps=bool(args.fuse_steps))
    flops = plan.flops()

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        tb.tasp_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        plan.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plan.run()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    # the same K calls once more, each bracketed by HIP events on the launch stream: the median
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in ev:
        e0.record()
        plan.run()
        e1.record()
    torch.cuda.synchronize()
    per_call = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    ms_median = per_call[len(per_call) // 2] if len(per_call) % 2 else 0.5 * (per_call[len(per_call) // 2 - 1] + per_call[len(per_call) // 2])

    # per-kernel durations, HIP events around every launch on the launch stream (same work again)
    n_prof = max(1, min(args.steps, 5))
    attn_ms = merge_ms = other_ms = 0.0
    attn_n = merge_n = 0
    for _ in range(n_prof):
        pr = plan.profile()
        attn_ms += pr.attn_ms
        merge_ms += pr.merge_ms
        other_ms += pr.other_ms
        attn_n += pr.attn_launches
        merge_n += pr.merge_launches
    is_bf16 = w.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if is_bf16 else PEAK_FP32_TFLOPS
    attn_avg_ms = attn_ms / max(attn_n, 1)
    # a launch = one step of Algorithm 3; the average launch does 1/launches of the call's flops
    # whatever the order or the schedule (totals over totals)
    flops_per_launch = flops / max(attn_n // n_prof, 1)
    achieved = flops_per_launch / (attn_avg_ms * 1e-3) / 1e12
    # HBM bytes per attention launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by
    # the copy-kernel calibration); the figures live in paper_2509_26541_amd/hbm_traffic.json, the
    # summaries they come from in profiles/
    # (null when the kernel source has changed since they were taken: the file records its hash)
    traffic = None
    tpath = os.path.join(ROOT, "paper_2509_26541_amd", "hbm_traffic.json")
    if os.path.exists(tpath) and args.batch == 1 and args.nodes <= 1 and args.order == "tasp" and args.fuse_merge and not args.fuse_steps:   # what was profiled
        import hashlib
        with open(os.path.join(ROOT, "paper_2509_26541_amd", "csrc", "attn_bf16.hip"), "rb") as f:
            sha = hashlib.sha256(f.read()).hexdigest()[:16]
        with open(tpath) as f:
            rec = json.load(f).get(w.name, {})
        if rec.get("attn_bf16_hip_sha16") == sha:
            traffic = rec.get("attn_bytes_per_launch")
    roofline = {
        "bound": "mfma" if is_bf16 else "alu", "kernel": "attn_bf16_kernel" if is_bf16 else "attn_fp32_kernel",
        "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": traffic,
        "avg_launch_ms": attn_avg_ms, "launches_per_call": attn_n // n_prof,
    }
    # the vector issue port, the pipe that actually bounds the bf16 kernel (above all at d = 64)
    roofline_valu = None
    if is_bf16:
        vp = valu_peak_tflops(w.d)
        roofline_valu = {"bound": "valu", "kernel": "attn_bf16_kernel", "achieved": achieved, "peak": vp, "unit": "TFLOP/s",
                         "frac": achieved / vp, "port_cycles": PORT_CYCLES, "per_tile_and_wavefront": TILE_MIX[w.d],
                         "port_cycles_measured": measure_port_cycles(tb)}
    def merge_stats(ms_total, launches, calls):
        # update_out_lse: per (row, head) read 2(4d+4) and write 4d+4 bytes; rows merged per call =
        # all rows of every task of steps 1..N-1
        bytes_per_rh = 3 * (4 * w.d + 4)
        rows_heads = 0
        for step in range(1, w.n_ranks):
            for qb in range(2 if w.mask_mode == wl.ZIGZAG_CAUSAL else 1):
                if sched.step_segments(w.S, w.mask_mode, step, qb, order=order):
                    rows_heads += (w.L // (2 if w.mask_mode == wl.ZIGZAG_CAUSAL else 1)) * w.Hq
        gbs = args.batch * rows_heads * bytes_per_rh / (ms_total / calls * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": "merge_kernel", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": gbs / PEAK_HBM_GBS, "ms_per_call": ms_total / calls, "launches_per_call": launches // calls}

    merge = merge_stats(merge_ms, merge_n, n_prof) if merge_n else None

    # the same call in the other merge mode
    other = None
    if not args.no_other_mode:
        alt = tb.ChunkAttnPlan(sched, qd, kd, vd, w.mask_mode, order=order, fuse_merge=not bool(args.fuse_merge))
        for _ in range(max(1, args.warmup)):
            alt.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            alt.run()
        torch.cuda.synchronize()
        alt_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        other = {"fuse_merge": int(not bool(args.fuse_merge)), "ms_per_step": alt_ms,
                 "value": flops / (alt_ms * 1e-3) / 1e12}
        if merge is None:
            a_ms, a_n = 0.0, 0
            for _ in range(n_prof):
                pr = alt.profile()
                a_ms += pr.merge_ms
                a_n += pr.merge_launches
            if a_n:
                merge = merge_stats(a_ms, a_n, n_prof)
        del alt

    # all steps in one launch (no per-step launch, set-up or merge); reported beside `value`, which
    # stays the step-by-step form with a merge after every block
    single = None
    if is_bf16 and not args.no_other_mode:
        try:
            one = tb.ChunkAttnPlan(sched, qd, kd, vd, w.mask_mode, order=order, fuse_steps=True)
            for _ in range(max(1, args.warmup)):
                one.run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                one.run()
            torch.cuda.synchronize()
            one_ms = (time.perf_counter() - t0) * 1e3 / args.steps
            single = {"fuse_steps": 1, "ms_per_step": one_ms, "value": flops / (one_ms * 1e-3) / 1e12,
                      "frac_of_bf16_mfma_peak": flops / (one_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
            del one
        except tb.TaspError as e:                 # more segments than the single launch takes
            single = {"fuse_steps": 1, "error": str(e)}

    def event_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    # what the matrix pipe of this box sustains with nothing else in the loop (clock under load included)
    calib_flops = tb.tasp_calibration_mfma(2000)
    mfma_peak = calib_flops / (event_ms(lambda: tb.tasp_calibration_mfma(2000), 3) * 1e-3) / 1e12

    # N partial pairs merged in one pass against the fold of the pairwise kernel (same buffers)
    merge_many = None
    if not args.no_other_mode:
        n_parts = w.n_ranks
        po = [torch.randn((w.L, w.Hq, w.d), dtype=torch.float32, device=dev) for _ in range(n_parts)]
        pl = [torch.randn((w.L, w.Hq), dtype=torch.float32, device=dev) for _ in range(n_parts)]
        oo, ol = torch.empty_like(po[0]), torch.empty_like(pl[0])
        unit = w.L * w.Hq * (4 * w.d + 4)

        def fold():
            for i in range(1, n_parts):
                tb.tasp_lse_merge(po[0], pl[0], po[i], pl[i])

        many_ms = event_ms(lambda: tb.tasp_lse_merge_many(po, pl, oo, ol), 3)
        fold_ms = event_ms(fold, 3)
        merge_many = {"n_parts": n_parts, "ms": many_ms, "GB/s": (n_parts + 1) * unit / (many_ms * 1e-3) / 1e9,
                      "pairwise_fold_ms": fold_ms, "pairwise_fold_GB/s": 3 * (n_parts - 1) * unit / (fold_ms * 1e-3) / 1e9}
        del po, pl, oo, ol

    # the backward pass of the same call (same schedule and order), timed the same way
    backward = None
    if is_bf16 and not args.no_backward:
        out_f, lse_f = plan.run()
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed + 104729)
        dout = torch.randn(qd.shape, generator=gen, device=dev, dtype=torch.float32).to(qd.dtype)
        def time_bwd(aux, fuse_steps=False):
            pl = tb.ChunkAttnBwdPlan(sched, qd, kd, vd, out_f, lse_f, dout, w.mask_mode, order=order, aux_stream=aux,
                                     fuse_steps=fuse_steps)
            for _ in range(max(1, args.warmup)):
                pl.run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                pl.run()
            torch.cuda.synchronize()
            return pl, (time.perf_counter() - t0) * 1e3 / args.steps

        # one stream, and the dk/dv kernels on a second stream beside the dq kernels
        bplan, one_ms = time_bwd(None)
        two_ms = fs_ms = None
        if not args.no_other_mode:                 # profiler runs: one kind of launch only
            aux_plan, two_ms = time_bwd(torch.cuda.Stream())
            del aux_plan
            try:                                   # all steps in one dq and one dk/dv launch
                fs_plan, fs_ms = time_bwd(None, fuse_steps=True)
                del fs_plan
            except tb.TaspError:
                fs_ms = None
        b_ms = one_ms if two_ms is None else min(one_ms, two_ms)
        bp = bplan.profile()
        b_flops = bplan.flops()                  # 2.5 x forward: five products
        backward = {
            "value": b_flops / (b_ms * 1e-3) / 1e12, "unit": "TFLOP/s", "ms_per_step": b_ms, "flops_per_call": b_flops,
            "ms_one_stream": one_ms, "ms_two_streams": two_ms,
            "single_launch": None if fs_ms is None else {"ms_per_step": fs_ms, "value": b_flops / (fs_ms * 1e-3) / 1e12},
            "frac_of_bf16_mfma_peak": b_flops / (b_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            # executed matrix work: the dq kernel forms three products per (query, key) pair (1.5 x the
            # forward's flops), the dk/dv kernel four (2 x): both recompute the scores
            "dq_kernel": {"avg_launch_ms": bp.dq_ms / max(bp.dq_launches, 1), "launches_per_call": bp.dq_launches,
                          "executed_TFLOP/s": 1.5 * flops / (bp.dq_ms * 1e-3) / 1e12},
            "dkv_kernel": {"avg_launch_ms": bp.dkv_ms / max(bp.dkv_launches, 1), "launches_per_call": bp.dkv_launches,
                           "executed_TFLOP/s": 2.0 * flops / (bp.dkv_ms * 1e-3) / 1e12},
            "other_ms": bp.other_ms,
        }
        del bplan, dout

    value = flops / (ms_per_step * 1e-3) / 1e12
    line = {
        "metric": "per-rank chunked-attention TFLOP/s on 1 MI355X", "value": value, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if is_bf16 else "f32", "data": "synthetic",
        "frac_of_bf16_mfma_peak": value / PEAK_BF16_TFLOPS if is_bf16 else None,
        "measured_mfma_only": {"value": mfma_peak, "unit": "TFLOP/s", "frac_of_it": value / mfma_peak if is_bf16 else None,
                               "what": "tasp_calibration_mfma: only v_mfma_f32_32x32x16_bf16, operands in registers"},
        "config": {"workload": w.name, "n_ranks": w.n_ranks, "rank": w.rank, "S": w.S, "L": w.L, "Hq": w.Hq,
                   "Hkv": w.Hkv, "d": w.d, "mask": "zigzag_causal" if w.mask_mode else "full",
                   "order": args.order, "rings": sched.n_rings, "batch": args.batch, "fuse_merge": int(args.fuse_merge), "fuse_steps": int(args.fuse_steps), "flops_per_call": flops},
        "roofline": roofline,
        "roofline_valu": roofline_valu,
        "ms_per_step_median_events": ms_median,
        "merge": merge,
        "ms_breakdown": {"attn": attn_ms / n_prof, "merge": merge_ms / n_prof, "cast": other_ms / n_prof},
        "other_merge_mode": other,
        "single_launch": single,
        "merge_many": merge_many,
        "backward": backward,
    }
    del plan, qd, kd, vd
    torch.cuda.empty_cache()
    if not args.grid and args.config == 2 and args.batch == 1 and not args.no_other_mode:
        line["other_workloads"] = other_workloads(tb, wl, torch, dev, order, args, t_start)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, q, k, v)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
