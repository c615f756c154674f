"""The library's host-side calibration steps (C ABI, no GPU) against the oracle:
bit-exact masks, schedule values, error codes."""
import ctypes as C
import math

import numpy as np
import pytest

import paper_2603_05503_amd as pkg
from oracle import calibration as cal


@pytest.mark.parametrize("seed", range(30))
def test_select_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    rows, nbk = int(rng.integers(1, 20)), int(rng.integers(1, 300))
    E = rng.dirichlet(np.full(nbk, float(rng.choice([0.05, 0.3, 1.0]))), size=rows).astype(np.float32)
    if seed % 3 == 0:  # ties
        E = (np.round(E * 16) / 16).astype(np.float32)
    eps = float(rng.choice([0.0, 0.3, 0.84, 0.99, 1.0, 1.5]))
    got = pkg.select_blocks(E, eps)
    want = cal.select_blocks(E, eps)
    assert got.dtype == np.uint8 and np.array_equal(got, want)


def test_select_shapes_and_hand_rows():
    E = np.array([[[0.1, 0.6, 0.05, 0.25], [0.25, 0.25, 0.25, 0.25]]], np.float32)
    assert pkg.select_blocks(E, 0.5).tolist() == [[[0, 1, 0, 0], [1, 1, 0, 0]]]
    assert pkg.select_blocks(E, 0.84).tolist() == [[[0, 1, 0, 1], [1, 1, 1, 1]]]
    tiny = np.array([1.0] + [2.0 ** -30] * 8, np.float32)
    assert pkg.select_blocks(tiny, 1.0 + 5 * 2.0 ** -30).sum() == 6  # running sum in double


@pytest.mark.parametrize("seed", range(10))
def test_vote_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    P = int(rng.integers(1, 70))
    masks = (rng.random((P, 3, 5, 7)) < rng.random()).astype(np.uint8) * rng.integers(1, 255, (P, 3, 5, 7)).astype(np.uint8)
    for rho in (0.0, 0.25, 0.5, 0.75, 1.0, float(rng.random())):
        assert np.array_equal(pkg.vote_masks(masks, rho), cal.vote(masks, rho)), rho


def test_incremental_vote_equals_the_stacked_vote():
    rng = np.random.default_rng(7)
    masks = (rng.random((9, 2, 6, 5)) < 0.5).astype(np.uint8) * rng.integers(1, 255, (9, 2, 6, 5)).astype(np.uint8)
    counts = np.zeros(masks.shape[1:], np.uint16)
    for m in masks:
        pkg.vote_accumulate(m, counts)
    assert np.array_equal(counts, (masks != 0).sum(axis=0))
    for rho in (0.0, 0.3, 0.5, 5 / 9, 0.9, 1.0):
        assert np.array_equal(pkg.vote_finish(counts, 9, rho), cal.vote(masks, rho)), rho
    lib = pkg.load_library()
    u8p, u16p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint16)
    full = np.full(3, 65535, np.uint16)
    one = np.ones(3, np.uint8)
    assert lib.calibatt_vote_accumulate(one.ctypes.data_as(u8p), 3, full.ctypes.data_as(u16p)) == -2 and (full == 65535).all()
    out = np.zeros(3, np.uint8)
    assert lib.calibatt_vote_finish(full.ctypes.data_as(u16p), 9, 3, 0.5, out.ctypes.data_as(u8p)) == -2  # count > prompts
    assert lib.calibatt_vote_finish(None, 9, 3, 0.5, out.ctypes.data_as(u8p)) == -1
    assert lib.calibatt_vote_finish(full.ctypes.data_as(u16p), 0, 3, 0.5, out.ctypes.data_as(u8p)) == -2


def test_schedule_matches_oracle_and_paper():
    A = pkg.schedule_base_level(32760)
    assert A == cal.schedule_base_level(32760)
    for T in (4, 50, 64):
        for t in range(T):
            assert pkg.epsilon_schedule(t, T, A, 0.99, 16.0) == cal.epsilon_schedule(t, T, A, 0.99, 16.0)
    assert pkg.epsilon_schedule(0, 50, A, 0.99, 16.0) == 0.99
    assert round(pkg.epsilon_schedule(49, 50, A, 0.99, 16.0), 2) == 0.84
    assert math.isnan(pkg.epsilon_schedule(0, 0, 0.8, 0.99, 16.0))


def test_schedule_constants_match_oracle():
    for regime in (0, 1):
        for N in (32760, 75600, 44776):
            assert pkg.schedule_constants(regime, N) == cal.schedule_constants(regime, N)
    lib = pkg.load_library()
    d = C.c_double()
    assert lib.calibatt_schedule_constants(2, 100, C.byref(d), C.byref(d), C.byref(d)) == -3
    assert lib.calibatt_schedule_constants(0, 0, C.byref(d), C.byref(d), C.byref(d)) == -2
    assert lib.calibatt_schedule_constants(0, 100, None, C.byref(d), C.byref(d)) == -1


@pytest.mark.parametrize("seed", range(6))
def test_flag_heads_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    n, H = int(rng.integers(1, 9)), int(rng.integers(1, 50))
    s = rng.uniform(0.6, 1.0, (n, H)).astype(np.float32)
    s[:, 0] = np.float32(0.87)  # a head that sits on the threshold (as fp32) on every prompt
    flags, mean = pkg.flag_heads(s, 0.87)
    want_flags, want_mean = cal.flag_heads(s, 0.87)
    assert np.array_equal(flags, want_flags) and np.array_equal(mean, want_mean)
    lib = pkg.load_library()
    assert lib.calibatt_flag_heads(None, 1, 1, 0.5, flags.ctypes.data_as(C.POINTER(C.c_uint8)), None) == -1
    assert lib.calibatt_flag_heads(s.ctypes.data_as(C.POINTER(C.c_float)), 0, 1, 0.5, flags.ctypes.data_as(C.POINTER(C.c_uint8)), None) == -2


def test_select_with_nan_energies_is_defined():
    # the comparator is a total order: NaN entries sort by their bit patterns, nothing is undefined, and rows
    # without NaN keep their exact masks
    E = np.array([[0.5, np.nan, 0.3, 0.2], [0.4, 0.3, 0.2, 0.1]], np.float32)
    m = pkg.select_blocks(E, 0.6)
    assert m.shape == (2, 4) and set(np.unique(m)) <= {0, 1}
    assert m[1].tolist() == cal.select_blocks(E[1:2], 0.6)[0].tolist()


def test_errors():
    lib = pkg.load_library()
    f32p, u8p = C.POINTER(C.c_float), C.POINTER(C.c_uint8)
    e = np.zeros(4, np.float32)
    m = np.zeros(4, np.uint8)
    ep, mp = e.ctypes.data_as(f32p), m.ctypes.data_as(u8p)
    assert lib.calibatt_select_blocks(None, 1, 4, 0.5, mp) == -1
    assert lib.calibatt_select_blocks(ep, 1, 4, 0.5, None) == -1
    assert lib.calibatt_select_blocks(ep, -1, 4, 0.5, mp) == -2
    assert lib.calibatt_select_blocks(ep, 1, 0, 0.5, mp) == -2
    assert lib.calibatt_select_blocks(ep, 1, 4, float("nan"), mp) == -2
    assert lib.calibatt_select_blocks(ep, 0, 4, 0.5, mp) == 0
    assert lib.calibatt_vote_masks(None, 1, 4, 0.5, mp) == -1
    assert lib.calibatt_vote_masks(mp, 0, 4, 0.5, mp) == -2
    assert lib.calibatt_vote_masks(mp, 1, 4, float("nan"), mp) == -2
    one = C.c_void_p(16)
    g = lib.calibatt_block_energy
    assert g(None, one, one, 1, 1, 8, 64, 64, 64, 1.0, None) == -1
    assert g(one, one, None, 1, 1, 8, 64, 64, 64, 1.0, None) == -1
    assert g(one, one, one, 1, 0, 8, 64, 64, 64, 1.0, None) == -2
    assert g(one, one, one, 1, 1, 8, 96, 64, 64, 1.0, None) == -3
    assert g(one, one, one, 1, 1, 8, 64, 32, 64, 1.0, None) == -3
    assert g(one, one, one, 1, 1, 10_000_000, 64, 64, 64, 1.0, None) == -3  # partial sums exceed LDS
