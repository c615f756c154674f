"""The build-time check of the kernel that addresses registers by name (csrc/check_named_regs.py):
planted violations in a piece of device assembly are reported, clean code and other kernels are not."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _checker():
    path = os.path.join(ROOT, "paper_2603_05503_amd", "csrc", "check_named_regs.py")
    spec = importlib.util.spec_from_file_location("check_named_regs", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _function(name, body):
    return f"\t.type\t{name},@function\n{name}:\n" + "".join(f"\t{line}\n" for line in body) + ".Lfunc_end0:\n"


KERNEL = "_ZN12calibatt_dev25sparse_attn_fwd_il_kernelILi128ELi128ELi128ELb0ENS_4Bf16EEEvPKt"
OTHER = "_ZN12calibatt_dev22sparse_attn_fwd_kernelILi128ELi128ELi128ELb0ENS_4Bf16EEEvPKt"
CLEAN = [
    "v_add_u32_e32 v5, v71, v3",
    "s_waitcnt vmcnt(0)",
    ";;#ASMSTART",
    "v_mfma_f32_32x32x16_bf16 a[0:15], a[64:67], v[72:75], a[0:15]",
    "v_accvgpr_write_b32 a88, v1",
    ";;#ASMEND",
    "v_lshlrev_b64 v[10:11], 2, v[12:13]",
]


def test_clean_kernel_passes():
    mod = _checker()
    assert mod.check(_function(KERNEL, CLEAN)) == []


def test_planted_violations_are_reported():
    mod = _checker()
    limit = mod.KERNELS["sparse_attn_fwd_il_kernel"]
    for bad in ("v_accvgpr_write_b32 a0, v19",          # the compiler parks a value in an AGPR
                "v_accvgpr_read_b32 v2, a0",
                f"v_mov_b32_e32 v{limit}, v1",           # an arch VGPR that belongs to the named range
                f"v_lshlrev_b64 v[{limit - 1}:{limit}], 2, v[2:3]",
                "scratch_store_dword off, v3, s0"):      # a spill
        problems = mod.check(_function(KERNEL, CLEAN + [bad]))
        assert len(problems) == 1 and bad.split()[0] in problems[0], bad


def test_other_kernels_are_not_policed():
    mod = _checker()
    assert mod.check(_function(OTHER, ["v_accvgpr_write_b32 a0, v19", "v_mov_b32_e32 v200, v1"])) == []
