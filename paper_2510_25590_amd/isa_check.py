"""Static check of the hand-pipelined global loads in the GEMM kernels' machine code.

csrc/gemm.hip issues its pipeline loads as inline assembly and waits for them by hand with `s_waitcnt vmcnt(N)`.
The compiler does not know that such a load writes its destination registers later than the point where the
instruction stands.  That is only correct while the generated code leaves those registers alone between the load and
the wait that covers it: no copy (a spill to an accumulation register or a move would copy stale data), no other
read, no other write.  Register pressure can make the compiler break that rule without any warning, and the result is
a kernel that reads or writes through corrupted registers.  This module compiles the file to assembly and proves the
rule on the control-flow graph of every `gemm_bf16_kernel` instantiation; the build fails otherwise.

Model: loads complete in issue order.  Every destination register of an asm load is "pending" with an age = number
of vector-memory loads issued after it.  `s_waitcnt vmcnt(N)` lands every register whose age is at least N.  At a
join the state is the union of the predecessors' pending sets with the smaller age.  Any instruction that names a
pending register is a violation (the load's own address operand excepted).
"""
from __future__ import annotations

import os
import re
import subprocess
import tempfile

_REG_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_REG_ONE = re.compile(r"\bv(\d+)\b")
_LABEL = re.compile(r"^(\.LBB\d+_\d+):")
_VMCNT = re.compile(r"vmcnt\((\d+)\)")


def _regs(text: str) -> set[int]:
    out: set[int] = set()
    for a, b in _REG_RANGE.findall(text):
        out.update(range(int(a), int(b) + 1))
    for a in _REG_ONE.findall(text):
        out.add(int(a))
    return out


def _kernel_bodies(asm: str, name_part: str):
    """Yields (mangled name, lines) of every function whose name contains name_part."""
    lines = asm.splitlines()
    i = 0
    while i < len(lines):
        m = re.match(r"^(_Z\w+):", lines[i])
        if m and name_part in m.group(1):
            j = i + 1
            while j < len(lines) and not lines[j].startswith(".Lfunc_end"):
                j += 1
            yield m.group(1), lines[i + 1:j]
            i = j
        i += 1


def _blocks(lines):
    """Splits a function into basic blocks: list of (label or None, [(instr, in_asm)], successors by label / fallthrough)."""
    blocks, cur, label, in_asm = [], [], None, False
    for raw in lines:
        s = raw.strip()
        if not s or s.startswith(";") and not s.startswith(";;#ASM"):
            continue
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = _LABEL.match(s)
        if m:
            if cur or label is not None:
                blocks.append([label, cur, None])
            label, cur = m.group(1), []
            continue
        if s.startswith("."):
            continue
        instr = s.split(";")[0].strip()
        if not instr:
            continue
        cur.append((instr, in_asm))
        op = instr.split()[0]
        if op.startswith("s_cbranch") or op == "s_branch" or op == "s_endpgm":
            blocks.append([label, cur, None])
            label, cur = None, []
    if cur or label is not None:
        blocks.append([label, cur, None])
    index = {b[0]: k for k, b in enumerate(blocks) if b[0] is not None}
    for k, b in enumerate(blocks):
        succ = []
        last = b[1][-1][0] if b[1] else ""
        op = last.split()[0] if last else ""
        if op == "s_endpgm":
            pass
        elif op == "s_branch":
            succ.append(index[last.split()[1]])
        else:
            if op.startswith("s_cbranch"):
                succ.append(index[last.split()[1]])
            if k + 1 < len(blocks):
                succ.append(k + 1)
        b[2] = succ
    return blocks


def _transfer(state: dict[int, int], block, where: str, errors: list[str]) -> dict[int, int]:
    st = dict(state)
    for instr, in_asm in block[1]:
        op = instr.split()[0]
        if op == "s_waitcnt":
            m = _VMCNT.search(instr)
            if m:
                n = int(m.group(1))
                st = {r: a for r, a in st.items() if a < n}
            continue
        is_vmem_load = op.startswith("global_load") or op.startswith("buffer_load") or op.startswith("flat_load") or op.startswith("scratch_load")
        named = _regs(instr)
        if in_asm and op == "global_load_dwordx4":
            operands = instr[len(op):].split(",")
            dest, rest = _regs(operands[0]), _regs(",".join(operands[1:]))
            bad = (rest - dest) & st.keys() | dest & st.keys()
            if bad:
                errors.append(f"{where}: '{instr}' names registers of loads still in flight: v{sorted(bad)}")
            st = {r: a + 1 for r, a in st.items()}
            for r in dest:
                st[r] = 0
            continue
        bad = named & st.keys()
        if bad:
            errors.append(f"{where}: '{instr}' names registers of loads still in flight: v{sorted(bad)}")
            for r in bad:          # report once
                st.pop(r)
        if is_vmem_load:
            st = {r: a + 1 for r, a in st.items()}
    return st


def check_function(name: str, lines, unroll: int = 0) -> list[str]:
    """Data flow over (block, last step run).
    unroll = 0: every path of the control-flow graph is followed.
    unroll = n: the K loop is unrolled n times and its step blocks (those that hold both asm loads and MFMAs) run
    in their order in the text, step 0 first, when the source guarantees that.  Block merging by the compiler can
    leave edges in the graph that would skip or repeat a step; a path that enters a step block out of order cannot
    run and is not followed."""
    blocks = _blocks(lines)
    if not blocks:
        return [f"{name}: no code found"]
    short = name[:60]

    def has(b, pred):
        return any(pred(i, a) for i, a in b[1])
    steps = [k for k, b in enumerate(blocks)
             if has(b, lambda i, a: a and i.startswith("global_load_dwordx4")) and has(b, lambda i, a: i.startswith("v_mfma"))]
    if unroll and len(steps) != unroll:
        return [f"{short}: expected {unroll} K-step blocks (asm loads and MFMAs), found {len(steps)}: the check does not know this shape"]
    step_id = {k: n for n, k in enumerate(steps)} if unroll else {}

    errors: list[str] = []
    seen_err: set[str] = set()
    entry: dict[tuple[int, int], dict[int, int]] = {(0, -1): {}}
    work = [(0, -1)]
    rounds = 0
    reached_steps: set[int] = set()
    while work:
        rounds += 1
        if rounds > 200000:
            return [f"{short}: analysis did not converge"]
        k, tag = work.pop()
        errs: list[str] = []
        out = _transfer(entry[(k, tag)], blocks[k], f"{short} block {blocks[k][0] or k} (after step {tag})", errs)
        for e in errs:
            if e not in seen_err:
                seen_err.add(e)
                errors.append(e)
        out_tag = step_id.get(k, tag)
        if k in step_id:
            reached_steps.add(k)
        last = blocks[k][1][-1][0].split()[0] if blocks[k][1] else ""
        if last == "s_endpgm" and out:
            e = f"{short}: loads into v{sorted(out)} may still be in flight at s_endpgm"
            if e not in seen_err:
                seen_err.add(e)
                errors.append(e)
        for s in blocks[k][2]:
            if unroll and s in step_id and step_id[s] != (out_tag + 1) % unroll:
                continue   # out of order: not a path of the program
            old = entry.get((s, out_tag))
            if old is None:
                new = dict(out)
            else:
                new = dict(old)
                for r, a in out.items():
                    new[r] = min(a, old[r]) if r in old else a
            if new != old:
                entry[(s, out_tag)] = new
                work.append((s, out_tag))
    if unroll and len(reached_steps) != unroll:
        errors.append(f"{short}: only {len(reached_steps)} of {unroll} K-step blocks are reachable in order")
    return errors


def check_gemm(hipcc: str, flags: list[str], source: str) -> None:
    """Compiles `source` to gfx950 assembly and checks every gemm_bf16_kernel; raises RuntimeError on a violation."""
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm.s")
        proc = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", source, "-o", out], capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed emitting assembly for the load check:\n" + proc.stderr)
        asm = open(out).read()
    n = 0
    problems: list[str] = []
    for name, lines in _kernel_bodies(asm, "gemm_bf16_kernel"):
        n += 1
        text = "\n".join(lines)
        m = re.search(r"; ScratchSize: (\d+)", asm[asm.index(name + ":"):])
        if m and int(m.group(1)) != 0:
            problems.append(f"{name[:60]}: uses {m.group(1)} bytes of scratch memory (its accesses share the load counter)")
        if "global_load_dwordx4" not in text:
            problems.append(f"{name[:60]}: no pipeline loads found")
        problems += check_function(name, lines)
    if n == 0:
        problems.append("no gemm_bf16_kernel instantiation found in the assembly")
    if problems:
        raise RuntimeError("GEMM pipeline-load check failed:\n  " + "\n  ".join(problems[:20]))
