"""Static check of the gfx950 assembly that hipcc produces for the kernels whose LDS reads are
written as inline assembly with hand-placed ``s_waitcnt lgkmcnt`` (tbn_linear_stream.hip,
tbn_linear_mfma.hip, tbn_conv_mfma.hip).

Such a read hands its destination registers to the compiler as if they were already filled; the
data arrives later, and the source only promises it after the wait that covers the read.  That
is sound exactly if, on every path, no instruction between the read and that wait touches the
destination registers (a register copy, a spill, a reuse for something else).  This module
walks the control-flow graph of each kernel, keeps the in-order queue of pending LDS
operations, retires entries at every ``s_waitcnt`` that carries an lgkmcnt, and reports

  * any instruction that names a register with a read still pending,
  * any scalar memory load while reads are pending (scalar loads share the counter but return
    out of order, so a non-zero count would no longer name the reads that have landed),
  * reads still pending at ``s_endpgm``.

Usage: ``python -m paper_2407_12075_amd.asm_check`` compiles the sources with ``-S`` and checks
them (exit status 1 on a finding); ``check_asm_text`` is the entry point for tests.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from typing import Dict, List, Optional, Tuple

_REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")
_LABEL = re.compile(r"^([.\w$]+):")
_LGKM = re.compile(r"lgkmcnt\((\d+)\)")


def _regs(text: str) -> frozenset:
    out = set()
    for m in _REG.finditer(text):
        kind = m.group(1)
        if m.group(2) is not None:
            out.add((kind, int(m.group(2))))
        else:
            out.update((kind, r) for r in range(int(m.group(3)), int(m.group(4)) + 1))
    return frozenset(out)


def _split_kernels(asm: str) -> Dict[str, List[str]]:
    """Instruction lines (labels included) of every function that ends in s_endpgm."""
    kernels: Dict[str, List[str]] = {}
    name: Optional[str] = None
    body: List[str] = []
    for raw in asm.splitlines():
        line = raw.split(";", 1)[0].rstrip()
        if not line.strip():
            continue
        m = _LABEL.match(line)
        if m and not line.startswith(".L") and not line.startswith("\t"):
            name, body = m.group(1), []
            continue
        if name is None:
            continue
        s = line.strip()
        if s.startswith(".") and not _LABEL.match(s):
            if s.startswith(".end_amdhsa_kernel") or s.startswith(".size") or s.startswith(".section"):
                if any("s_endpgm" in b for b in body):
                    kernels[name] = body
                name = None
            continue
        body.append(s)
    return kernels


def _simm_lgkm(ins: str) -> Optional[int]:
    """lgkmcnt of an s_waitcnt, None if it does not constrain that counter."""
    m = _LGKM.search(ins)
    if m:
        return int(m.group(1))
    m = re.match(r"s_waitcnt\s+(0x[0-9a-fA-F]+|\d+)\s*$", ins)
    if m:   # raw immediate, gfx9 layout: lgkmcnt in bits 11:8
        v = (int(m.group(1), 0) >> 8) & 15
        return None if v == 15 else v
    return None


def check_kernel(name: str, body: List[str], max_states: int = 200000) -> List[str]:
    labels = {}
    ins: List[str] = []
    for line in body:
        m = _LABEL.match(line)
        if m:
            labels[m.group(1)] = len(ins)
        else:
            ins.append(line)
    findings: List[str] = []
    seen = set()
    # state: tuple of pending LDS operations in issue order; an entry is the frozenset of
    # destination registers (empty for LDS writes)
    stack: List[Tuple[int, tuple]] = [(0, ())]
    block_starts = set(labels.values())
    steps = 0
    while stack:
        i, pend = stack.pop()
        while True:
            if i >= len(ins):
                break
            if i in block_starts:
                key = (i, pend)
                if key in seen:
                    break
                seen.add(key)
            steps += 1
            if steps > max_states * 50:
                findings.append(f"{name}: state space too large, check abandoned")
                return findings
            text = ins[i]
            op = text.split()[0]
            busy = frozenset().union(*pend) if pend else frozenset()
            if op == "s_waitcnt":
                n = _simm_lgkm(text)
                if n is not None and len(pend) > n:
                    pend = pend[len(pend) - n:] if n else ()
            elif op.startswith("ds_"):
                operands = text[len(op):]
                touched = _regs(operands)
                if touched & busy:
                    findings.append(f"{name}: '{text}' uses registers of a pending LDS read (instruction {i})")
                if op.startswith("ds_read") or op.startswith("ds_load"):
                    dst = _regs(operands.split(",")[0])
                    pend = pend + (dst,)
                else:
                    pend = pend + (frozenset(),)
                if len(pend) > 15:   # the 4-bit counter is full: the wave could not issue before the oldest landed
                    pend = pend[-15:]
            else:
                if busy and _regs(text[len(op):]) & busy:
                    findings.append(f"{name}: '{text}' touches registers of a pending LDS read (instruction {i})")
                if (op.startswith("s_load") or op.startswith("s_buffer_load")) and any(pend):
                    findings.append(f"{name}: scalar load '{text}' while LDS reads are pending (instruction {i})")
            if op == "s_endpgm":
                if any(pend):
                    findings.append(f"{name}: LDS reads pending at s_endpgm")
                break
            if op == "s_branch":
                i = labels[text.split()[1]]
                continue
            if op.startswith("s_cbranch"):
                stack.append((labels[text.split()[1]], pend))
            i += 1
        if len(seen) > max_states:
            findings.append(f"{name}: state space too large, check abandoned")
            break
    # one finding per offending instruction is enough
    return sorted(set(findings))


def check_asm_text(asm: str) -> Tuple[List[str], List[str]]:
    """(names of the kernels checked, findings)."""
    kernels = _split_kernels(asm)
    findings: List[str] = []
    for name, body in kernels.items():
        findings += check_kernel(name, body)
    return sorted(kernels), findings


def compile_to_asm(src: str) -> str:
    from . import build as hip_build
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = [hip_build.HIPCC, *hip_build.FLAGS, "--cuda-device-only", "-S", src, "-o", out]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc -S failed for {src}:\n{res.stderr}")
        return open(out).read()


CHECKED_SOURCES = ("tbn_linear_block.hip", "tbn_linear_stream.hip", "tbn_linear_mfma.hip", "tbn_conv_mfma.hip")


def main() -> int:
    from . import build as hip_build
    bad = 0
    for src in CHECKED_SOURCES:
        names, findings = check_asm_text(compile_to_asm(os.path.join(hip_build.CSRC, src)))
        print(f"{src}: {len(names)} kernels, {len(findings)} findings")
        for f in findings[:40]:
            print("  " + f)
        bad += len(findings)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
