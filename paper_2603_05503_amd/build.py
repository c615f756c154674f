"""Builds libcalibatt.so (host pattern compiler + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libcalibatt.so")
PROBE_PATH = os.path.join(PKG_DIR, "mfma_peak_probe.bin")  # stand-alone executable, see csrc/mfma_peak_probe.hip

SOURCES = ["compile_pattern.cpp", "anchor_map.cpp", "calibration.cpp", "skiplist.cpp", "sparse_attn_fwd.hip"]

# Packed fp32 VALU forms are switched off for all device code.
HIP_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Wno-inline-asm",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = True, extra_flags=()) -> str:
    import importlib.util
    import tempfile

    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    # --save-temps leaves the device assembly of this very compilation in the working directory:
    # the kernels that name registers by hand are checked on it (csrc/check_named_regs.py).
    cmd = [hipcc(), *HIP_FLAGS, *extra_flags, "--save-temps", "-I", os.path.join(ROOT, "include"), "-I", CSRC, *srcs,
           "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    with tempfile.TemporaryDirectory() as tmp:
        subprocess.run(cmd, check=True, cwd=tmp)
        spec = importlib.util.spec_from_file_location("check_named_regs", os.path.join(CSRC, "check_named_regs.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        asm = os.path.join(tmp, "sparse_attn_fwd-hip-amdgcn-amd-amdhsa-gfx950.s")
        problems = mod.check(open(asm).read())
    if problems:
        os.remove(LIB_PATH)
        raise RuntimeError("named-register kernels: the compiler used a reserved register:\n" + "\n".join(problems[:20]))
    probe = [hipcc(), *[f for f in HIP_FLAGS if f not in ("-fPIC", "-shared")], "-Wno-unused-value",
             os.path.join(CSRC, "mfma_peak_probe.hip"), "-o", PROBE_PATH]
    if verbose:
        print(" ".join(probe), flush=True)
    subprocess.run(probe, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
