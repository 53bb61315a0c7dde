"""Static check of this package's own gfx950 code: scalar registers that a vector-memory instruction reads.

On this architecture a vector-memory instruction that takes a scalar register (its base address) reads a stale
value if a vector-ALU instruction wrote that register fewer than five wait states before it; the hardware does
not interlock the case.  The compiler pads the loads it emits itself, but it does not look into an `asm`
statement, and it restores spilled scalars with `v_readlane` right in front of their use.  The kernels here issue
their streaming loads from `asm` statements, so every build is checked:

  * `compile_to_isa` turns one of the package's device sources into ISA text (`hipcc -S`, the device pass only);
  * `hazards` walks that text backwards from every vector-memory instruction with scalar operands, over all
    control-flow predecessors, and reports each vector-ALU write of one of those scalars within five wait states.

A second rule has the same root: the destination registers of a load issued from an `asm` statement hold nothing
until the hand-written wait, so they must not be copied in between.  The compiler keeps to that as long as it has
registers; once it spills vector registers to scratch it may save exactly such a register, and the kernel computes
with what was there before the load (seen once with a tighter occupancy bound: wrong numbers, no fault).
`spilled_asm_kernels` lists the kernels that spill a vector register straight after one of their `asm` loads wrote it.

`build()` runs both checks on every device source and fails on a finding; tests call them too.
"""
from __future__ import annotations

import os
import re
import subprocess
from typing import Dict, List, Tuple

WAIT_STATES = 5

_VMEM = ("global_", "buffer_", "flat_", "scratch_")
_LABEL = re.compile(r"^([A-Za-z_.$][\w.$]*):$")
_SREG = re.compile(r"\bs\[(\d+):(\d+)\]|\bs(\d+)\b")


def _sregs(text: str) -> set:
    out = set()
    for m in _SREG.finditer(text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _operands(text: str) -> List[str]:
    parts = text.split(None, 1)
    return [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []


def _valu_scalar_writes(text: str) -> set:
    """Scalar registers a vector-ALU instruction writes (lane reads, compares into a scalar pair, carry outputs)."""
    op = text.split()[0]
    if not op.startswith("v_"):
        return set()
    ops = _operands(text)
    out = set()
    if ops and re.fullmatch(r"s\[\d+:\d+\]|s\d+", ops[0]):
        out |= _sregs(ops[0])
    carry = ("_co_" in op or op.startswith(("v_addc", "v_subb", "v_subbrev", "v_div_scale", "v_mad_u64_u32", "v_mad_i64_i32")))
    if carry and len(ops) > 1 and re.fullmatch(r"s\[\d+:\d+\]|s\d+", ops[1]):
        out |= _sregs(ops[1])
    return out


def _wait_states(text: str) -> int:
    if text.startswith("s_nop"):
        return int(text.split()[1], 0) + 1
    return 1


def hazards(isa_text: str) -> List[Tuple[int, str, int, str, int]]:
    """Findings as (line of the write, write, line of the memory instruction, memory instruction, wait states between)."""
    ins: List[Tuple[int, str]] = []
    labels: Dict[str, int] = {}
    for n, raw in enumerate(isa_text.splitlines(), 1):
        s = raw.split(";")[0].strip()
        if not s:
            continue
        m = _LABEL.match(s)
        if m:
            labels[m.group(1)] = len(ins)
            continue
        if s.startswith("."):
            continue
        ins.append((n, s))
    preds: List[List[int]] = [[] for _ in ins]
    for i, (_, s) in enumerate(ins):
        op = s.split()[0]
        falls = op not in ("s_branch", "s_endpgm", "s_setpc_b64")
        if op == "s_branch" or op.startswith("s_cbranch"):
            tgt = labels.get(s.split()[1])
            if tgt is not None and tgt < len(ins):
                preds[tgt].append(i)
        if falls and i + 1 < len(ins):
            preds[i + 1].append(i)
    found = []
    for i, (ln, s) in enumerate(ins):
        op = s.split()[0]
        if not op.startswith(_VMEM):
            continue
        need = set()
        for o in _operands(s):
            if re.fullmatch(r"s\[\d+:\d+\]|s\d+", o.split()[0] if o else ""):
                need |= _sregs(o.split()[0])
        if not need:
            continue
        # backwards over every path, until five wait states lie between
        stack = [(j, 0) for j in preds[i]]
        seen: Dict[int, int] = {}
        while stack:
            j, ws = stack.pop()
            if ws >= WAIT_STATES or seen.get(j, WAIT_STATES) <= ws:
                continue
            seen[j] = ws
            lnj, t = ins[j]
            hit = _valu_scalar_writes(t) & need
            if hit:
                found.append((lnj, t, ln, s, ws))
                continue
            ws2 = ws + _wait_states(t)
            for k in preds[j]:
                stack.append((k, ws2))
    return found


def _vregs(text: str) -> set:
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def spilled_asm_kernels(isa_text: str) -> List[Tuple[str, List[int]]]:
    """(kernel, registers) for every kernel that spills a vector register whose last writer, going back from the
    spill in program order, is a vector-memory load inside an asm statement (no wait in between)."""
    lines = isa_text.splitlines()
    kernel_at: List[str] = []
    in_asm_at: List[bool] = []
    cur, in_asm = None, False
    for raw in lines:
        s = raw.strip()
        m = re.match(r"^([A-Za-z_][\w$]*):", raw)
        if m and not raw.startswith("."):
            cur = m.group(1)
        if s.startswith(";;#ASMSTART"):
            in_asm = True
        elif s.startswith(";;#ASMEND"):
            in_asm = False
        kernel_at.append(cur)
        in_asm_at.append(in_asm)
    found: Dict[str, set] = {}
    for i, raw in enumerate(lines):
        s = raw.strip()
        if not s.startswith("scratch_store") or "Spill" not in s:
            continue
        ops = _operands(s.split(";")[0])
        regs = _vregs(ops[1] if len(ops) > 1 else "")
        for j in range(i - 1, max(i - 2000, -1), -1):
            if kernel_at[j] != kernel_at[i] or not regs:
                break
            t = lines[j].split(";")[0].strip() if not lines[j].strip().startswith(";;#") else ""
            if not t or t.endswith(":") or t.startswith("."):
                continue
            op = t.split()[0]
            if op == "s_waitcnt" and "vmcnt" in t:
                break                                   # whatever was in flight has been waited for (or counted) here
            if op.startswith(("v_", "ds_read", "ds_load")) or (op.startswith(_VMEM) and "load" in op and "lds" not in op):
                dst = _vregs(_operands(t)[0]) if _operands(t) else set()
                hit = dst & regs
                if hit:
                    if in_asm_at[j] and op.startswith(_VMEM):
                        found.setdefault(kernel_at[i], set()).update(hit)
                    regs = regs - hit
    return [(k, sorted(v)) for k, v in found.items()]


def compile_to_isa(source: str, out_path: str, hipcc: str, flags: List[str]) -> str:
    cmd = [hipcc, *flags, "-S", "--offload-device-only", "-o", out_path, source]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    with open(out_path) as f:
        return f.read()


def check_source(source: str, build_dir: str, hipcc: str, flags: List[str]) -> List[tuple]:
    """Findings of both checks for one device source (empty: clean)."""
    out = os.path.join(build_dir, os.path.basename(source) + ".s")
    text = compile_to_isa(source, out, hipcc, flags)
    return hazards(text) + [(0, f"spills v{regs}", 0, f"kernel {name}: destinations of its asm loads", -1)
                            for name, regs in spilled_asm_kernels(text)]
