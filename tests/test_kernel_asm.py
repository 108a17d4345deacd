"""The generated code of the bf16 attention kernel keeps the hand-placed LDS waits valid (CPU only:
hipcc cross-compiles to assembly without a GPU)."""
import os
import re
import shutil

import pytest

from tests import asm_checks

pytestmark = pytest.mark.skipif(shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is None,
                                reason="hipcc not found")


@pytest.fixture(scope="module")
def attn_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "attn_bf16.s"
    return asm_checks.compile_to_asm("attn_bf16.hip", str(out))


@pytest.fixture(scope="module")
def bwd_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "attn_bwd_bf16.s"
    return asm_checks.compile_to_asm("attn_bwd_bf16.hip", str(out))


def test_checker_flags_a_planted_violation():
    ok = [(1, "ds_read_b128 v[4:7], v1 offset:0"), (2, "s_waitcnt lgkmcnt(0)"), (3, "v_mov_b32_e32 v9, v4")]
    early = [(1, "ds_read_b128 v[4:7], v1 offset:0"), (2, "v_mov_b32_e32 v9, v4"), (3, "s_waitcnt lgkmcnt(0)")]
    younger = [(1, "ds_read_b128 v[4:7], v1"), (2, "ds_read_b128 v[8:11], v1"), (3, "s_waitcnt lgkmcnt(1)"),
               (4, "v_add_f32_e32 v0, v4, v5"), (5, "v_add_f32_e32 v0, v8, v9")]
    assert asm_checks.in_flight_violations(ok) == []
    assert [b[0] for b in asm_checks.in_flight_violations(early)] == [2]
    assert [b[0] for b in asm_checks.in_flight_violations(younger)] == [5]


def test_attention_kernels_found(attn_asm):
    ks = asm_checks.kernels(attn_asm)
    names = [k for k in ks if "attn_bf16_kernel" in k]
    assert len(names) == 4, names      # d = 128; d = 64 with 8 and 12 wavefronts, the former also with persistent workgroups
    for k in names:
        ops = [s.split()[0] for _, s in ks[k]]
        assert sum(o.startswith("v_mfma_f32_32x32x16_bf16") for o in ops) >= 32
        assert any(o == "ds_read_b64_tr_b16" for o in ops) and any(o == "ds_read_b128" for o in ops)
        assert not any(o.startswith("flat_") for o in ops), k
        # tile fetches: buffer loads straight into LDS.  Their asm statement asks for the descriptor
        # and the moving offset in scalar registers; the compiler has been seen to hand over a vector
        # register there (a wavefront-uniform value it had decided to keep in one), which assembles
        # in this text form and is no valid instruction, so every one of them is checked.
        loads = [s for _, s in ks[k] if s.startswith("buffer_load_dwordx4")]
        assert len(loads) >= 8, (k, len(loads))
        for s in loads:
            assert re.fullmatch(r"buffer_load_dwordx4 v\d+, s\[\d+:\d+\], s\d+ offen lds", s), (k, s)


def test_bench_tile_mix_matches_the_generated_code(attn_asm):
    """bench.py prices the vector issue port with the instruction mix of one key tile; the counts it
    uses are those of the generated code (a few vector instructions of slack for compiler versions)."""
    import bench
    for name, ins in asm_checks.kernels(attn_asm).items():
        if "attn_bf16_kernel" not in name:
            continue
        d = 128 if "ILi128E" in name else 64
        mix, want = asm_checks.tile_body_mix(ins), bench.TILE_MIX[d]
        assert mix["mfma"] == want["mfma"] and mix["lds_kib"] == want["lds_kib"], (name, mix)
        assert abs(mix["exp"] - want["exp"]) <= 1 and abs(mix["valu"] - want["valu"]) <= 4, (name, mix)


def test_no_register_of_a_pending_lds_read_is_touched(attn_asm):
    for name, ins in asm_checks.kernels(attn_asm).items():
        if "attn_bf16_kernel" not in name:
            continue
        bad = asm_checks.in_flight_violations(ins)
        assert bad == [], "%s: %d instructions touch registers of LDS reads still in flight, first: %r" % (
            name, len(bad), bad[:3])


def test_no_spills_in_the_loop(attn_asm):
    """No spills at all in the d = 128 kernel and the d = 64 kernels of the plain grid.  The variant
    with persistent workgroups (ELb1EEE) may park values between two work items, but nothing inside
    the loop over key tiles (there the innermost loop, nesting depth 2)."""
    rep = [r for r in asm_checks.spill_report(attn_asm) if "attn_bf16_kernel" in r[0]]
    assert len(rep) == 4
    for name, spills, scratch in rep:
        if "ELb1EEE" in name:
            assert spills <= 64, (name, spills)
        else:
            assert spills == 0 and scratch == 0, (name, spills, scratch)
    assert asm_checks.scratch_in_loops(attn_asm, "ELb0EEEvNS_10AttnLaunch") == []
    assert asm_checks.scratch_in_loops(attn_asm, "ELb1EEEvNS_10AttnLaunch", min_depth=2) == []


def _is_lds_load(s):
    return (s.startswith("global_load_lds_dwordx4") or s.startswith("global_load_lds_dword ")
            or (s.startswith("buffer_load_dwordx4") and s.endswith(" lds")))


def _m0_misuse(instructions):
    """Instructions that name m0 outside the one pattern the direct global->LDS loads use (their asm
    statement: s_mov_b32 m0, <sgpr> / s_nop 0 / global_load_lds_dwordx4, global_load_lds_dword or
    buffer_load_dwordx4 .. lds),
    and such loads without it."""
    ins = [(line, s) for line, s in instructions if not s.endswith(":")]
    bad = []
    for k, (line, s) in enumerate(ins):
        op = s.split()[0]
        if re.search(r"\bm0\b", s):
            ok = (op == "s_mov_b32" and s.split()[1].rstrip(",") == "m0" and k + 2 < len(ins)
                  and ins[k + 1][1] == "s_nop 0" and _is_lds_load(ins[k + 2][1]))
            if not ok:
                bad.append((line, s))
        if _is_lds_load(s) and not (k >= 2 and ins[k - 2][1].startswith("s_mov_b32 m0,") and ins[k - 1][1] == "s_nop 0"):
            bad.append((line, s))
    return bad


def test_m0_checker_flags_planted_uses():
    good = [(1, "s_mov_b32 m0, s4"), (2, "s_nop 0"), (3, "global_load_lds_dwordx4 v1, s[2:3]")]
    assert _m0_misuse(good) == []
    assert _m0_misuse([(1, "s_mov_b32 m0, s4"), (2, "s_nop 0"), (3, "buffer_load_dwordx4 v1, s[4:7], s9 offen lds")]) == []
    assert [b[0] for b in _m0_misuse([(3, "buffer_load_dwordx4 v1, s[4:7], s9 offen lds")])] == [3]
    assert [b[0] for b in _m0_misuse(good + [(4, "v_readlane_b32 s5, v2, m0")])] == [4]
    assert [b[0] for b in _m0_misuse([(1, "s_mov_b32 m0, s4"), (2, "v_mov_b32_e32 v0, v1"), (3, "global_load_lds_dwordx4 v1, s[2:3]")])] == [1, 3]


def test_m0_belongs_to_the_direct_loads_only(attn_asm, bwd_asm):
    """The asm statement of the direct global->LDS load writes m0 without declaring it.  That is
    sound as long as the compiler itself never keeps a value in m0: in the generated code of every
    kernel that uses these loads, m0 appears in that statement's three instructions and nowhere else."""
    for asm in (attn_asm, bwd_asm):
        for name, ins in asm_checks.kernels(asm).items():
            if any(_is_lds_load(s) for _, s in ins):
                assert _m0_misuse(ins) == [], (name, _m0_misuse(ins)[:3])


# ---------------------------------------------------------------- backward kernels (compiler-scheduled)
def test_backward_kernels_shape_and_register_budget(bwd_asm):
    """Six instantiations (the dk/dv kernel also split by query head); each reads its LDS tiles with LDS instructions (no flat loads: the address
    space was inferred), fills them with direct global->LDS loads, fits the 256 registers that let two
    wavefronts share a SIMD, and keeps register spills out of the loop that holds the matrix
    instructions."""
    import re
    ks = {k: v for k, v in asm_checks.kernels(bwd_asm).items() if "bwd_dq_kernel" in k or "bwd_dkv_kernel" in k}
    assert len(ks) == 6, list(ks)
    budget = dict((m.group(1), int(m.group(2))) for m in re.finditer(
        r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)", bwd_asm))
    for name, ins in ks.items():
        ops = [s.split()[0] for _, s in ins]
        mf = [i for i, o in enumerate(ops) if o.startswith("v_mfma_f32_32x32x16_bf16")]
        assert len(mf) >= 24, (name, len(mf))
        assert "ds_read_b64_tr_b16" in ops and "ds_read_b128" in ops
        assert "global_load_lds_dwordx4" in ops or "buffer_load_dwordx4" in ops
        for s in (s for _, s in ins if s.startswith("buffer_load_dwordx4")):      # descriptor and offset in scalar registers
            assert re.fullmatch(r"buffer_load_dwordx4 v\d+, s\[\d+:\d+\], (s\d+|0) offen lds", s), (name, s)
        assert not any(o.startswith("flat_load") or o.startswith("flat_store") for o in ops), name
        assert budget[name] <= 256, (name, budget[name])
        spills = [i for i, o in enumerate(ops) if o.startswith("scratch_")]
        assert all(i < mf[0] or i > mf[-1] for i in spills), (name, "spill inside the matrix loop")
    for name, n_spill, _ in asm_checks.spill_report(bwd_asm):
        if name in ks:
            assert n_spill <= 4, (name, n_spill)


def _vmcnt_waits_in_matrix_loop(ins):
    """(line, text) of every s_waitcnt that names vmcnt between the first and the last matrix
    instruction, except the hand-written one on the tile fetch (vmcnt(0) alone, followed by the
    barrier)."""
    ops = [s for _, s in ins if not s.endswith(":")]
    lines = [l for l, s in ins if not s.endswith(":")]
    mf = [i for i, s in enumerate(ops) if s.startswith("v_mfma_")]
    bad = []
    for i in range(mf[0], mf[-1]):
        if ops[i].startswith("s_waitcnt") and "vmcnt" in ops[i]:
            if ops[i] == "s_waitcnt vmcnt(0)" and any(o.startswith("s_barrier") for o in ops[i + 1:i + 4]):
                continue
            bad.append((lines[i], ops[i]))
    return bad


def test_vmcnt_checker_flags_planted_waits():
    loop = [(1, "v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]"), (2, "s_waitcnt vmcnt(0)"), (3, "s_barrier"),
            (4, "s_waitcnt lgkmcnt(2)"), (5, "v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]")]
    assert _vmcnt_waits_in_matrix_loop(loop) == []
    planted = loop[:3] + [(4, "s_waitcnt vmcnt(1) lgkmcnt(2)")] + loop[4:]
    assert _vmcnt_waits_in_matrix_loop(planted) == [(4, "s_waitcnt vmcnt(1) lgkmcnt(2)")]


def test_backward_loops_never_wait_on_vector_memory_by_themselves(bwd_asm):
    """The tile fetches of the dq and dk/dv kernels are direct global->LDS loads inside asm statements, waited
    for by a hand-written vmcnt(0) before the barrier.  The compiler does not see that wait: if it
    believes other loads (the stationary rows, lse, delta) are still on their way inside the loop,
    it waits for them there, and in hardware such a wait stalls on the fetch of the next tile.  So the
    matrix loop holds no vmcnt wait but the hand-written one."""
    ks = {k: v for k, v in asm_checks.kernels(bwd_asm).items() if "bwd_dkv_kernel" in k or "bwd_dq_kernel" in k}
    assert len(ks) == 6, list(ks)
    for name, ins in ks.items():
        assert _vmcnt_waits_in_matrix_loop(ins) == [], (name, _vmcnt_waits_in_matrix_loop(ins)[:3])
