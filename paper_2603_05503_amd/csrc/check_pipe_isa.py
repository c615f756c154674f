#!/usr/bin/env python3
"""Checks the compiled pipelined kernel: outside the generated instruction streams the compiler
must not touch the registers those streams own (v64-v255, a8-a255), must not use scratch memory,
and the kernel must be given the whole register file.

usage: check_pipe_isa.py <file.s>   (device assembly of sparse_attn_fwd.hip, hipcc -S --cuda-device-only)
Exit status 0 when all holds; prints what it found otherwise."""
import re
import sys

FIRST_OWNED_VGPR = 64
FIRST_OWNED_AGPR = 8


def check(text):
    lines = text.split("\n")
    try:
        start = next(i for i, l in enumerate(lines) if re.match(r"_ZN12calibatt_dev27sparse_attn_fwd_pipe_kernel.*:", l))
    except StopIteration:
        return ["pipelined kernel not found in the assembly"]
    end = next(i for i in range(start, len(lines)) if lines[i].strip().startswith("s_endpgm"))
    problems = []
    inasm = False
    for i in range(start, end):
        l = lines[i]
        if "#ASMSTART" in l:
            inasm = True
            continue
        if "#ASMEND" in l:
            inasm = False
            continue
        s = l.strip()
        if inasm or not s or s.startswith((";", ".")):
            continue
        regs = set()
        for m in re.finditer(r"\b([va])(\d+)\b", s):
            regs.add((m.group(1), int(m.group(2))))
        for m in re.finditer(r"\b([va])\[(\d+):(\d+)\]", s):
            regs.update((m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1))
        if any((c == "v" and r >= FIRST_OWNED_VGPR) or (c == "a" and r >= FIRST_OWNED_AGPR) for c, r in regs):
            problems.append(f"line {i + 1}: compiler instruction touches an owned register: {s}")
    meta = "\n".join(lines[end:end + 120])
    for key, want in (("NumVgprs", 256), ("NumAgprs", 256), ("ScratchSize", 0)):
        m = re.search(rf"; {key}: (\d+)", meta)
        if not m or int(m.group(1)) != want:
            problems.append(f"{key} is {m.group(1) if m else 'missing'}, expected {want}")
    return problems


if __name__ == "__main__":
    found = check(open(sys.argv[1]).read())
    for f in found:
        print(f)
    sys.exit(1 if found else 0)
