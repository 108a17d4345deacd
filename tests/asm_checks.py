"""Static checks on the assembly hipcc generates for the bf16 attention kernel.

The kernel issues its LDS operand reads as inline assembly and waits for them by hand (s_waitcnt
lgkmcnt(N) placed in front of the matrix instruction that consumes the fragment).  The compiler does
not know that the destination registers of such a read are still "in flight" after the read has been
issued; the source keeps them live up to the wait, so a correct build never touches them in between.
This module re-derives that property from the generated code: it follows every path through the
basic blocks, keeps the list of LDS instructions that may still be outstanding (LDS instructions of
a wavefront complete in order, a wait for "at most N outstanding" retires all but the youngest N;
the fragment stream of the loop runs across its back edge) and reports every instruction that reads
or writes a register of an outstanding read.  It also reports register spills.
"""
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2509_26541_amd", "csrc")


def compile_to_asm(source, out_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S", "--cuda-device-only",
           "-x", "hip", os.path.join(CSRC, source), "-o", out_path]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr[-4000:])
    with open(out_path) as f:
        return f.read()


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"(?<![\w\[:])v(\d+)\b", text):
        out.add(int(m.group(1)))
    return out


def kernels(asm):
    """{kernel symbol: list of (line number, text)} for every kernel of the module: its instructions
    and, as entries that end with a colon, the labels of its basic blocks."""
    out, name = {}, None
    for i, line in enumerate(asm.split("\n")):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name = m.group(1)
            out[name] = []
            continue
        if name is None:
            continue
        if line.startswith("\t.end_amdhsa_kernel") or line.startswith(".Lfunc_end"):
            name = None
            continue
        s = line.split(";")[0].strip()
        if not s or (s.startswith(".") and not s.endswith(":")):
            continue
        out[name].append((i + 1, s))
    return out


def _blocks(instructions):
    """Basic blocks of an instruction list (labels are entries that end with a colon) with successors."""
    blocks, cur = [], {"label": None, "ins": []}
    for line, s in instructions:
        if s.endswith(":"):
            blocks.append(cur)
            cur = {"label": s[:-1], "ins": []}
            continue
        cur["ins"].append((line, s))
        op = s.split()[0]
        if op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm", "s_setpc_b64"):
            blocks.append(cur)
            cur = {"label": None, "ins": []}
    blocks.append(cur)
    by_label = {b["label"]: k for k, b in enumerate(blocks) if b["label"] is not None}
    for k, b in enumerate(blocks):
        succ = []
        last = b["ins"][-1][1] if b["ins"] else ""
        op = last.split()[0] if last else ""
        target = last.split()[-1] if last else ""
        if op == "s_branch":
            succ = [by_label[target]] if target in by_label else []
        elif op in ("s_endpgm", "s_setpc_b64"):
            succ = []
        else:
            if op.startswith("s_cbranch") and target in by_label:
                succ.append(by_label[target])
            if k + 1 < len(blocks):
                succ.append(k + 1)
        b["succ"] = succ
    return blocks


def _walk(ins, pending, bad):
    """One basic block: `pending` = LDS instructions that may be outstanding at its entry, oldest
    first, each (destination registers, line of issue).  Returns the list at its exit."""
    pending = list(pending)
    for line, s in ins:
        op = s.split()[0]
        operands = s[len(op):].split(",")
        if op.startswith("ds_read") or op.startswith("ds_bpermute") or op.startswith("ds_permute"):
            src = set().union(*[_regs(x) for x in operands[1:]]) if len(operands) > 1 else set()
            for regs, issued in pending:
                if regs & src:
                    bad.add((line, s, issued))
            pending.append((frozenset(_regs(operands[0])), line))
            continue
        if op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load") or op == "s_memtime":
            pending.append((frozenset(), line))      # counts towards lgkmcnt, returns no vector register
            continue
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", s)
            if m:
                n = int(m.group(1))
                pending = pending[len(pending) - n:] if n > 0 else []
            elif not re.search(r"(vmcnt|expcnt)\(", s):
                pending = []                    # numeric form: treat as a full wait
            continue
        touched = _regs(s[len(op):])
        for regs, issued in pending:
            if regs & touched:
                bad.add((line, s, issued))
    return pending[-64:]


def in_flight_violations(instructions):
    """Instructions that touch a register of an LDS read that may not have landed yet, along every
    path through the code: the list of possibly outstanding reads at the entry of a basic block is
    the merge over its predecessors, aligned at the youngest end (a wait for "at most N
    outstanding" retires all but the youngest N), iterated until nothing changes."""
    blocks = _blocks(instructions)
    entry = [None] * len(blocks)
    entry[0] = []
    work = [0]
    while work:
        k = work.pop()
        out = _walk(blocks[k]["ins"], entry[k], set())
        for t in blocks[k]["succ"]:
            if entry[t] is None:
                merged = list(out)
            else:
                old, n = entry[t], max(len(entry[t]), len(out))
                merged = []
                for pos in range(n):              # position counted from the youngest end
                    a = old[len(old) - 1 - pos] if pos < len(old) else (frozenset(), 1 << 30)
                    b = out[len(out) - 1 - pos] if pos < len(out) else (frozenset(), 1 << 30)
                    merged.append((a[0] | b[0], min(a[1], b[1])))
                merged.reverse()
            if entry[t] is None or merged != entry[t]:
                entry[t] = merged
                work.append(t)
    bad = set()
    for k, b in enumerate(blocks):
        if entry[k] is not None:
            _walk(b["ins"], entry[k], bad)
    return sorted(bad)


def tile_body_mix(instructions):
    """Instruction mix of one 64-key tile on the common path of the attention kernel's key loop: the
    instructions between two consecutive barriers of the loop (the first such stretch that holds at
    least 16 matrix instructions, after the barriers of the set-up), following the fall-through of
    every conditional branch except s_cbranch_vccz, which is taken when no row's maximum has grown.
    Returns {"mfma", "valu" (vector instructions other than matrix and exponential), "exp",
    "lds_kib" (KiB returned by LDS reads to a wavefront), "other"}."""
    ins = list(instructions)
    bars = [k for k, (_, s) in enumerate(ins) if s == "s_barrier"]
    seg = None
    for j in range(3, len(bars) - 1):
        if sum(1 for _, s in ins[bars[j]:bars[j + 1]] if s.startswith("v_mfma")) >= 16:
            seg = ins[bars[j] + 1:bars[j + 1] + 1]
            break
    assert seg is not None
    label_at = {s[:-1]: k for k, (_, s) in enumerate(seg) if s.endswith(":")}
    mix = {"mfma": 0, "valu": 0, "exp": 0, "lds_kib": 0.0, "other": 0}
    k = 0
    while k < len(seg):
        s = seg[k][1]
        op = s.split()[0]
        if op == "s_cbranch_vccz" and label_at.get(s.split()[-1], -1) > k:
            k = label_at[s.split()[-1]]
            continue
        k += 1
        if s.endswith(":"):
            continue
        if op.startswith("v_mfma"):
            mix["mfma"] += 1
        elif op.startswith("v_exp"):
            mix["exp"] += 1
        elif op.startswith("v_"):
            mix["valu"] += 1
        else:
            mix["other"] += 1
            if op == "ds_read_b128":
                mix["lds_kib"] += 1.0
            elif op.startswith("ds_read_b64"):
                mix["lds_kib"] += 0.5
    return mix


def spill_report(asm):
    """(kernel, vgpr_spill_count, private_segment_fixed_size) per kernel from the metadata block."""
    out = []
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)\n(?:.*\n)*?\s+\.vgpr_spill_count:\s+(\d+)", asm):
        out.append((m.group(1), int(m.group(3)), int(m.group(2))))
    return out


def scratch_in_loops(asm, kernel_substring, min_depth=1):
    """(kernel, block label) of every basic block that the compiler marks as part of a loop nested at
    least `min_depth` deep and that holds a scratch (spill) instruction, for kernels whose symbol
    contains `kernel_substring`."""
    out, name, label, deep = [], None, None, False
    for line in asm.split("\n"):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, label, deep = (m.group(1) if kernel_substring in m.group(1) else None), None, False
            continue
        if name is None:
            continue
        if line.startswith(".Lfunc_end"):
            name = None
            continue
        m = re.match(r"^(\.LBB\d+_\d+):(.*)", line)
        if m:
            label = m.group(1)
            depths = [int(d) for d in re.findall(r"Depth[= ](\d+)", m.group(2))]
            deep = bool(depths) and max(depths) >= min_depth
            continue
        if deep and line.strip().startswith("scratch_"):
            out.append((name, label))
    return out
