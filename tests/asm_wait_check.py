"""Checker for loads issued from inline assembly in the compiled gfx950 kernels (host-side, text only).

A load written as inline assembly is invisible to the compiler's bookkeeping of outstanding memory operations: the
compiler believes the destination registers hold their value as soon as the statement has been issued, inserts no
wait of its own, and is free to hand those registers to other values once the source stops using them.  The source
therefore has to place every wait by hand.  This module reads the assembly hipcc writes for a kernel and walks every
path through it, keeping the queue of outstanding vector-memory operations, and reports each instruction that reads
or writes a register while an assembly load into that register may still be in flight.

Model (gfx9 family): vector-memory operations retire in issue order among loads, `s_waitcnt vmcnt(n)` leaves at most
the newest n outstanding.  Stores and loads may retire out of order with respect to each other, so while a store is
outstanding only `vmcnt(0)` is taken to retire anything.  At most 63 operations can be outstanding.
"""
from __future__ import annotations

import re

_VMEM = re.compile(r"^(global_|buffer_|scratch_|flat_)")
_LABEL = re.compile(r"^(\.L\w+):")
_KERNEL = re.compile(r"^(_Z\w+|[A-Za-z_]\w*):\s*(;.*)?$")
_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def _vgprs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1) is not None:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return frozenset(out)


def split_kernels(asm_text):
    """{symbol: [(line number, text)]} for every function body of an assembly file."""
    kernels, name = {}, None
    for ln, t in enumerate(asm_text.split("\n"), 1):
        if t.startswith(".Lfunc_end"):
            name = None
            continue
        m = _KERNEL.match(t)
        if m and not t.startswith(".") and not t.startswith("\t"):
            name = m.group(1)
            kernels[name] = []
            continue
        if name is not None:
            kernels[name].append((ln, t))
    return kernels


def parse(body):
    """Instructions of one function: list of (line, mnemonic + operands, issued from inline assembly) and label map."""
    ins, labels, in_asm = [], {}, False
    for ln, t in body:
        s = t.strip()
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = _LABEL.match(t)
        if m:
            labels[m.group(1)] = len(ins)
            continue
        s = s.split(";")[0].strip()
        if not s or s.startswith("."):
            continue
        ins.append((ln, s, in_asm))
    return ins, labels


def check(body):
    """Walk every path of one function.  Returns (violations, number of tracked loads); a violation is
    (line of the load, line of the instruction that touches its register too early, that instruction)."""
    ins, labels = parse(body)
    tracked = 0
    for _, s, a in ins:
        if a and s.startswith("global_load_dword") and "_lds_" not in s:
            tracked += 1
    violations = set()
    seen = set()
    work = [(0, ())]
    while work:
        pc, pending = work.pop()
        while pc < len(ins):
            key = (pc, pending)
            if key in seen:
                break
            seen.add(key)
            ln, s, a = ins[pc]
            op = s.split()[0]
            if op == "s_waitcnt":
                m = re.search(r"vmcnt\((\d+)\)", s)
                if m:
                    n = int(m.group(1))
                    if n == 0:
                        pending = ()
                    elif not any(kind == "S" for kind, _, _ in pending):
                        pending = pending[max(0, len(pending) - n):]
                elif re.fullmatch(r"s_waitcnt\s+(0x[0-9a-fA-F]+|\d+)", s):
                    raise ValueError(f"line {ln}: undecoded wait '{s}'")
                pc += 1
                continue
            touched = _vgprs(s)
            for kind, regs, at in pending:
                if regs and (touched & regs):
                    violations.add((at, ln, s))
            if _VMEM.match(op):
                if a and op.startswith("global_load_dword") and "_lds_" not in op:
                    entry = ("L", _vgprs(s.split(",")[0]), ln)
                elif "store" in op or "atomic" in op:
                    entry = ("S", frozenset(), ln)
                else:
                    entry = ("L", frozenset(), ln)
                pending = (pending + (entry,))[-63:]
            if op == "s_endpgm":
                break
            if op in ("s_setpc_b64", "s_swappc_b64"):
                raise ValueError(f"line {ln}: indirect branch, paths cannot be enumerated")
            if op == "s_branch" or op.startswith("s_cbranch"):
                target = s.split()[-1]
                if target not in labels:
                    raise ValueError(f"line {ln}: branch to unknown label {target}")
                if op == "s_branch":
                    pc = labels[target]
                    continue
                work.append((labels[target], pending))
            pc += 1
    return sorted(violations), tracked
