"""The pipelined kernel owns most of the register file by name; the compiler must stay out of
it.  The build verifies that on the real assembly; here the checker itself is tested on
synthetic assembly, and the committed generated header is checked against its generator."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_05503_amd", "csrc")


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(CSRC, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


KERNEL = "_ZN12calibatt_dev27sparse_attn_fwd_pipe_kernelILi128ELi128ELi128EEEvPKt:"
META = "; NumVgprs: 256\n; NumAgprs: 256\n; ScratchSize: 0\n"


def _asm(body, meta=META):
    return f"{KERNEL}\n{body}\n\ts_endpgm\n{meta}"


def test_checker_accepts_clean_code():
    chk = _load("check_pipe_isa")
    body = "\tv_mov_b32 v3, v5\n\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_bf16 a[128:143], a[32:35], v[192:195], a[128:143]\n\t;;#ASMEND\n\tv_accvgpr_write_b32 a1, v7"
    assert chk.check(_asm(body)) == []


def test_checker_flags_compiler_use_of_owned_registers():
    chk = _load("check_pipe_isa")
    for bad in ("v_mov_b32 v64, v5", "v_mov_b64 v[62:65], v[2:5]", "v_accvgpr_write_b32 a8, v1", "v_accvgpr_read_b32 v1, a200"):
        assert chk.check(_asm("\t" + bad)), bad


def test_checker_flags_register_budget_and_scratch():
    chk = _load("check_pipe_isa")
    assert chk.check(_asm("\ts_nop 0", META.replace("ScratchSize: 0", "ScratchSize: 16")))
    assert chk.check(_asm("\ts_nop 0", META.replace("NumAgprs: 256", "NumAgprs: 224")))
    assert chk.check("nothing here")


def test_generated_header_is_current(tmp_path):
    """attn_pipe_asm.h is what gen_pipe_asm.py writes."""
    gen = os.path.join(CSRC, "gen_pipe_asm.py")
    committed = open(os.path.join(CSRC, "attn_pipe_asm.h")).read()
    copy = tmp_path / "gen_pipe_asm.py"
    copy.write_text(open(gen).read())
    env = {k: v for k, v in os.environ.items() if k != "PIPE_GEN_EXP"}
    subprocess.run([sys.executable, str(copy)], check=True, env=env)
    assert (tmp_path / "attn_pipe_asm.h").read_text() == committed
