"""Check the compiled wave-specialised kernels for register traffic the compiler must not add.

The matrix blocks of csrc/ws_kernels.hip issue MFMAs and ring loads inside inline assembly,
so the compiler does not know that accumulators are still being written by the matrix pipeline
or that ring registers have loads in flight.  That is safe only while no instruction outside
the assembly blocks touches an accumulator register between a matrix block and the block that
drains the matrix pipeline, or a ring register (a destination of an in-assembly
`global_load_dwordx4`) between the first matrix block and the block holding `s_waitcnt vmcnt(0)`.
This script compiles the file to ISA and checks it, and also that none of these kernels spills a
vector register.

Usage: python -m paper_2602_23111_amd.lint_isa      (exit status 0 = clean)
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "ws_kernels.hip")


def _regs(tok: str) -> set[str]:
    m = re.match(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return {f"{m.group(1)}{i}" for i in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.match(r"([va])(\d+)$", tok)
    return {f"{m.group(1)}{m.group(2)}"} if m else set()


def lint_text(isa: str) -> list[str]:
    """Violations found in the ISA text, one line each (empty list = clean)."""
    problems = []
    kernels = list(re.finditer(r"^(_Z\w*_ws_kernel\w*):[^\n]*\n(.*?)\.Lfunc_end", isa, re.S | re.M))
    if not kernels:
        return ["no *_ws_kernel function found in the ISA"]
    for m in kernels:
        name, body = m.group(1), m.group(2).split("\n")
        ring, inasm = set(), False
        for line in body:
            if "ASMSTART" in line:
                inasm = True
            elif "ASMEND" in line:
                inasm = False
            elif inasm and "global_load_dwordx4" in line:
                ring |= _regs(line.split()[1].rstrip(","))
        if not ring:
            problems.append(f"{name}: no ring loads found inside assembly blocks")
            continue
        # Walk the text in order.  Accumulators are busy from an assembly block with MFMAs until an
        # assembly block that drains the matrix pipeline (four `s_nop 15` and no MFMA); ring registers
        # from the first matrix block (before it the compiler may still use a slot's registers: the
        # first fills do not touch every slot) until the assembly block with `s_waitcnt vmcnt(0)`.
        # (A loop body is laid out once; its drain precedes the code that reads the accumulators.)
        inasm = acc_busy = ring_busy = ring_done = False
        block = []
        for line in body:
            if "ASMSTART" in line:
                inasm, block = True, []
                continue
            if "ASMEND" in line:
                inasm = False
                text = "\n".join(block)
                if "v_mfma" in text:
                    acc_busy = True
                    ring_busy = ring_busy or not ring_done
                elif text.count("s_nop 15") >= 4:
                    acc_busy = False
                if "s_waitcnt vmcnt(0)" in text:
                    ring_busy, ring_done = False, True
                continue
            if inasm:
                block.append(line)
                continue
            text = line.strip()
            if not text or text[0] in ".;" or text.startswith("s_"):
                continue
            ops = text.replace(",", " ").split()
            used = set()
            for o in ops[1:]:
                used |= _regs(o)
            if acc_busy and ("accvgpr" in ops[0] or any(r.startswith("a") for r in used)):
                problems.append(f"{name}: accumulator register touched outside assembly: {text}")
            elif ring_busy and used & ring:
                problems.append(f"{name}: ring register touched outside assembly: {text}")
    # A spilled register in these kernels is a performance bug (every wave is given the register count of the
    # hungriest one, and the streaming loops have no slack for scratch traffic) and moves values through memory
    # behind the back of the in-flight loads above: the kernel metadata must report none.
    for m in re.finditer(r"\.name:\s+(\S*_ws_kernel\S*)(.*?)\.wavefront_size", isa, re.S):
        sp = re.search(r"\.vgpr_spill_count:\s+(\d+)", m.group(2))
        if sp and int(sp.group(1)) != 0:
            problems.append(f"{m.group(1)}: {sp.group(1)} vector registers spilled to scratch")
    return problems


def compile_isa() -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "ws.s")
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG, "csrc"), "-S",
               "--cuda-device-only", "-o", out, SRC]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc -S failed:\n" + res.stderr)
        return open(out).read()


if __name__ == "__main__":
    found = lint_text(compile_isa())
    for p in found:
        print(p)
    print("ws_kernels.hip ISA:", "clean" if not found else f"{len(found)} problem(s)")
    sys.exit(1 if found else 0)
