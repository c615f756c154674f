"""Host logic of the C-ABI library (no GPU): the C++ pattern compiler must equal
the integer oracle bit for bit, reject what the oracle rejects, and the shared
library must export every symbol the public header declares."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2603_05503_amd as pkg
from oracle import PatternError
from oracle import compile_pattern as oracle_compile
from oracle import pattern_sizes as oracle_sizes
from tests.test_pattern_oracle import REJECTED, check_against_worked_example, check_invariants
from workloads import make_workload, random_mask

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ARRAYS = ("row_ptr", "col_idx", "repeat_src", "work", "fan_ptr", "fan_dst")
KIND_TO_STATUS = {"range": -4, "chain": -5, "tail": -6}


def _lib_compile(mask, repeat, H, N, bq, bk, order):
    hp = pkg.compile_pattern(mask, repeat, H, N, bq, bk, order)
    d = {name: getattr(hp, name) for name in ARRAYS}
    d.update(nnz=hp.nnz, n_work=hp.n_work, n_repeat=hp.n_repeat, nbq=hp.nbq, nbk=hp.nbk, max_row=hp.max_row,
             n_groups=hp.n_groups, group_ptr=hp.group_ptr)
    return d


def _assert_equal(a, b):
    for name in ARRAYS:
        assert a[name].dtype == np.int32
        assert np.array_equal(a[name], b[name]), name
    for name in ("nnz", "n_work", "n_repeat", "nbq", "nbk", "n_groups"):
        assert a[name] == b[name], name
    assert a["group_ptr"].tolist() == b["group_ptr"].tolist()


def test_header_symbols_exported():
    header = open(os.path.join(ROOT, "include", "calibatt.h")).read()
    names = set(re.findall(r"^(?:int|double|const char \*)\s*(calibatt_\w+)\s*\(", header, flags=re.M))
    assert {"calibatt_pattern_sizes", "calibatt_compile_pattern", "calibatt_sparse_attn_fwd",
            "calibatt_anchor_map", "calibatt_anchor_attn_fwd", "calibatt_block_energy", "calibatt_select_blocks",
            "calibatt_vote_masks", "calibatt_vote_accumulate", "calibatt_vote_finish", "calibatt_epsilon_schedule", "calibatt_schedule_base_level",
            "calibatt_sparse_attn_fwd_strided", "calibatt_sparse_attn_fwd_ex", "calibatt_anchor_attn_fwd_strided", "calibatt_anchor_attn_fwd_split", "calibatt_select_blocks_device", "calibatt_block_energy_onepass", "calibatt_block_energy_workspace_bytes", "calibatt_vote_accumulate_device", "calibatt_anchor_split_plan", "calibatt_anchor_partner", "calibatt_spatial_similarity", "calibatt_spatial_similarity_static", "calibatt_encode_intervals", "calibatt_merge_intervals", "calibatt_share_timesteps", "calibatt_strerror", "calibatt_version"} <= names
    lib = ctypes.CDLL(pkg.library_path())
    for n in names:
        assert hasattr(lib, n), n
    assert pkg.version() >= 100
    assert "success" in pkg.strerror(0)


def test_library_worked_example():
    check_against_worked_example(_lib_compile)


@pytest.mark.parametrize("seed", range(60))
def test_library_matches_oracle_random(seed):
    rng = np.random.default_rng(1000 + seed)
    H = int(rng.integers(1, 5))
    bq, bk = int(rng.choice([4, 8, 16, 64])), int(rng.choice([4, 8, 16, 128]))
    N = int(rng.integers(1, 400))
    nbq, nbk = -(-N // bq), -(-N // bk)
    dens = float(rng.choice([0.0, 0.05, 0.3, 0.7, 1.0]))
    mask, repeat = random_mask(seed, H, nbq, nbk, dens, float(rng.choice([0, 0.1, 0.5])), tail_partial=(N % bq) != 0)
    mask = mask * rng.integers(1, 255, size=mask.shape).astype(np.uint8)
    if seed % 5 == 0:
        repeat = None
    for order in (0, 1, 2, 3, 4):
        a = _lib_compile(mask, repeat, H, N, bq, bk, order)
        b = oracle_compile(mask, repeat, H, N, bq, bk, order)
        _assert_equal(a, b)
        check_invariants(a, mask, repeat, H, N, bq, bk, order)
        assert a["max_row"] == (np.diff(b["row_ptr"]).max() if b["row_ptr"].size > 1 else 0)
    assert pkg.pattern_sizes(mask, repeat, H, N, bq, bk) == oracle_sizes(mask, repeat, H, N, bq, bk)


@pytest.mark.parametrize("name", ["tiny", "wan480", "mochi"])
def test_library_matches_oracle_named_configs(name):
    wl = make_workload(name, with_qkv=False, heads=None if name == "tiny" else 11)
    for order in (0, 1, 2, 3, 4):
        a = _lib_compile(wl.mask, wl.repeat, wl.H, wl.N, wl.block_q, wl.block_k, order)
        b = oracle_compile(wl.mask, wl.repeat, wl.H, wl.N, wl.block_q, wl.block_k, order)
        _assert_equal(a, b)


@pytest.mark.parametrize("rep,N,bq,kind", REJECTED)
def test_library_rejects_like_oracle(rep, N, bq, kind):
    mask = np.ones((1, 4, 4), dtype=np.uint8)
    repeat = np.array([rep], np.int32)
    with pytest.raises(PatternError):
        oracle_compile(mask, repeat, 1, N, bq, 8, 1)
    with pytest.raises(pkg.CalibattError) as e:
        pkg.compile_pattern(mask, repeat, 1, N, bq, 8, 1)
    assert e.value.status == KIND_TO_STATUS[kind]
    with pytest.raises(pkg.CalibattError) as e:
        pkg.pattern_sizes(mask, repeat, 1, N, bq, 8)
    assert e.value.status == KIND_TO_STATUS[kind]


def test_library_error_codes_raw_abi():
    lib = pkg.load_library()
    mask = np.ones(16, np.uint8)
    bufs = [np.zeros(32, np.int32) for _ in range(6)]
    from paper_2603_05503_amd.binding import _CPattern, _ptr

    cp = _CPattern()
    args = lambda m, order, cap: (
        m, None, 1, 32, 8, 8, order, _ptr(bufs[0], ctypes.c_int32), _ptr(bufs[1], ctypes.c_int32), cap,
        _ptr(bufs[2], ctypes.c_int32), _ptr(bufs[3], ctypes.c_int32), _ptr(bufs[4], ctypes.c_int32),
        _ptr(bufs[5], ctypes.c_int32), ctypes.byref(cp))
    m = _ptr(mask, ctypes.c_uint8)
    assert lib.calibatt_compile_pattern(*args(None, 1, 16)) == -1
    assert lib.calibatt_compile_pattern(*args(m, 7, 16)) == -3
    assert lib.calibatt_compile_pattern(*args(m, 1, 15)) == -7
    assert lib.calibatt_compile_pattern(*args(m, 1, 16)) == 0
    assert (cp.nnz, cp.n_work, cp.n_repeat, cp.nbq, cp.nbk, cp.max_row) == (16, 4, 0, 4, 4, 4)
    assert lib.calibatt_pattern_sizes(m, None, 0, 32, 8, 8, None, None, None) == -2
    assert lib.calibatt_pattern_sizes(m, None, 1, 32, 8, 8, None, None, None) == 0
    # forward: argument validation happens on the host before any GPU call
    assert cp.n_groups == 1 and list(cp.group_ptr)[:2] == [0, 4]
    cp.H, cp.N, cp.block_q, cp.block_k = 1, 32, 8, 8
    one = ctypes.c_void_p(16)
    fwd = lib.calibatt_sparse_attn_fwd
    assert fwd(None, one, one, one, 1, 1, 32, 64, 64, 64, ctypes.byref(cp), 1.0, None) == -1
    assert fwd(one, one, one, ctypes.c_void_p(32), 1, 1, 32, 48, 64, 64, ctypes.byref(cp), 1.0, None) == -3
    assert fwd(one, one, one, ctypes.c_void_p(32), 1, 1, 32, 64, 64, 64, ctypes.byref(cp), 1.0, None) == -8
    assert fwd(one, one, one, ctypes.c_void_p(32), 0, 1, 32, 64, 64, 64, ctypes.byref(cp), 1.0, None) == -2
    assert fwd(one, one, one, one, 1, 1, 32, 64, 64, 64, ctypes.byref(cp), 1.0, None) == -2  # out aliases q


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own, with warnings as errors."""
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "calibatt.h"\n'
                   "int main(void) {\n"
                   "  calibatt_fwd_options options;\n"
                   "  calibatt_pattern pattern;\n"
                   "  (void)options;\n"
                   "  (void)pattern;\n"
                   "  return calibatt_version() > 0 ? 0 : 1;\n"
                   "}\n")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)
