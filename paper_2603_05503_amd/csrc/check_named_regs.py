"""Build-time check of the kernels that address registers by name (attn_kernel_il.h).

Those kernels are compiled for a reduced number of arch VGPRs and use the registers above that
number, and all AGPRs, from inline assembly only.  The compiler does not know what those registers
hold; should it ever place a value of its own there (it may, for instance, park a VGPR in a free
AGPR instead of spilling it), the kernel would compute garbage or fault.  This script reads the
device assembly of the build and fails it when, inside such a kernel and outside the inline-asm
blocks, an instruction names an AGPR, an arch VGPR at or above the limit, or scratch memory.
"""
import re
import sys

KERNELS = {"sparse_attn_fwd_il_kernel": 72}  # kernel name fragment -> arch VGPRs left to the compiler


def check(text):
    problems = []
    in_asm = False
    limit = None
    func = None
    for ln, line in enumerate(text.splitlines(), 1):
        t = line.strip()
        if t.startswith(".type") and "@function" in t:
            func = t.split()[1].rstrip(",")
            limit = next((v for k, v in KERNELS.items() if k in func), None)
            in_asm = False
            continue
        if ";;#ASMSTART" in t:
            in_asm = True
            continue
        if ";;#ASMEND" in t:
            in_asm = False
            continue
        if limit is None or in_asm or not t or t[0] in ";.":
            continue
        code = t.split(";")[0]
        bad = any(int(m.group(1)) >= limit for m in re.finditer(r"\bv(\d+)\b", code))
        bad = bad or any(int(m.group(2)) >= limit for m in re.finditer(r"\bv\[(\d+):(\d+)\]", code))
        bad = bad or re.search(r"\ba\d+\b|\ba\[\d+", code) is not None or "scratch_" in code
        if bad:
            problems.append(f"{func}: line {ln}: {t}")
    return problems


if __name__ == "__main__":
    found = check(open(sys.argv[1]).read())
    print(f"{len(found)} problem(s)")
    for f in found[:20]:
        print(f)
    sys.exit(1 if found else 0)
