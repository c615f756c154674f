"""The library's host-side skip-list tools (C ABI, no GPU) against the oracle:
bit-exact interval words, merged masks, clusters; error codes."""
import ctypes as C

import numpy as np
import pytest

import paper_2603_05503_amd as pkg
from oracle import skiplist as sl
from workloads import random_mask


@pytest.mark.parametrize("seed", range(20))
def test_encode_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    H, nb = int(rng.integers(1, 4)), int(rng.integers(1, 80))
    N, blk = nb * 8 - int(rng.integers(0, 8)), 8
    nb = -(-N // blk)
    mask, repeat = random_mask(seed, H, nb, nb, float(rng.choice([0.0, 0.1, 0.5, 1.0])), float(rng.choice([0, 0.3])),
                               tail_partial=(N % blk) != 0)
    hp = pkg.compile_pattern(mask, repeat, H, N, blk, blk, 0)
    iv_ptr, iv = hp.encode_intervals()
    rows = mask.reshape(H * nb, nb).copy()
    rows[(repeat.reshape(-1) >= 0)] = 0  # repeated rows compile to empty lists
    want_ptr, want = sl.encode_intervals(rows)
    assert iv_ptr.dtype == np.int32 and iv.dtype == np.uint32
    assert np.array_equal(iv_ptr, want_ptr) and np.array_equal(iv, want)
    assert (sl.decode_intervals(iv_ptr, iv, nb) == (rows != 0)).all()


def test_encode_hand_worked_and_errors():
    row_ptr = np.array([0, 6, 6, 9], np.int32)
    col_idx = np.array([0, 1, 4, 6, 7, 8, 2, 3, 4], np.int32)
    iv_ptr, iv = pkg.encode_intervals(row_ptr, col_idx)
    assert iv_ptr.tolist() == [0, 4, 5, 7]
    assert iv.tolist() == [0, 4 | (2 << 16), 6 | (3 << 16), 6 << 16, 0, 2, 3 << 16]
    lib = pkg.load_library()
    i32p, u32p = C.POINTER(C.c_int32), C.POINTER(C.c_uint32)
    n = C.c_int64(0)
    rp = row_ptr.ctypes.data_as(i32p)
    assert lib.calibatt_encode_intervals(None, col_idx.ctypes.data_as(i32p), 3, None, None, 0, C.byref(n)) == -1
    assert lib.calibatt_encode_intervals(rp, col_idx.ctypes.data_as(i32p), -1, None, None, 0, C.byref(n)) == -2
    bad = np.array([0, 1, 4, 4, 7, 8, 2, 3, 4], np.int32)  # not strictly ascending
    assert lib.calibatt_encode_intervals(rp, bad.ctypes.data_as(i32p), 3, None, None, 0, C.byref(n)) == -2
    big = np.array([0, 1, 4, 6, 7, 70000, 2, 3, 4], np.int32)
    assert lib.calibatt_encode_intervals(rp, big.ctypes.data_as(i32p), 3, None, None, 0, C.byref(n)) == -2
    out_ptr, out = np.zeros(4, np.int32), np.zeros(3, np.uint32)
    assert lib.calibatt_encode_intervals(rp, col_idx.ctypes.data_as(i32p), 3, out_ptr.ctypes.data_as(i32p),
                                         out.ctypes.data_as(u32p), 3, C.byref(n)) == -7
    assert n.value == 7


@pytest.mark.parametrize("seed", range(20))
def test_merge_matches_oracle(seed):
    rng = np.random.default_rng(50 + seed)
    shape = (int(rng.integers(1, 4)), int(rng.integers(1, 30)), int(rng.integers(1, 60)))
    m = (rng.random(shape) < rng.random()).astype(np.uint8) * rng.integers(1, 255, shape).astype(np.uint8)
    for pct in (100, 99, 95, 90, 50, 1):
        got, w = pkg.merge_intervals(m, pct)
        want, w_want = sl.merge_mask(m, pct)
        assert w == w_want and np.array_equal(got, want), pct


def test_merge_in_place_and_errors():
    lib = pkg.load_library()
    u8p = C.POINTER(C.c_uint8)
    m = np.array([[1, 0, 0, 1, 0, 1, 1, 0, 0, 0, 1], [1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1]], np.uint8)
    want, _ = sl.merge_mask(m, 50)
    buf = m.copy()
    w = C.c_int32(0)
    assert lib.calibatt_merge_intervals(buf.ctypes.data_as(u8p), 2, 11, 50.0, buf.ctypes.data_as(u8p), C.byref(w)) == 0
    assert w.value == 1 and np.array_equal(buf, want)
    for pct in (0.0, -1.0, 100.5, float("nan")):
        assert lib.calibatt_merge_intervals(buf.ctypes.data_as(u8p), 2, 11, pct, buf.ctypes.data_as(u8p), None) == -2
    assert lib.calibatt_merge_intervals(None, 2, 11, 50.0, buf.ctypes.data_as(u8p), None) == -1
    assert lib.calibatt_merge_intervals(buf.ctypes.data_as(u8p), 2, 0, 50.0, buf.ctypes.data_as(u8p), None) == -2


@pytest.mark.parametrize("seed", range(12))
def test_sharing_matches_oracle(seed):
    rng = np.random.default_rng(80 + seed)
    T = int(rng.integers(1, 20))
    base = (rng.random((5, 9)) < 0.5).astype(np.uint8)
    masks = np.stack([np.where(rng.random(base.shape) < 0.02 * t, 1 - base, base) for t in range(T)])
    masks = masks * rng.integers(1, 255, masks.shape).astype(np.uint8)
    for tau in (0.0, 0.5, 0.8, 0.9, 0.97, 1.0):
        ids, shared = pkg.share_timesteps(masks, tau)
        want_ids, want_shared = sl.share_timesteps(masks, tau)
        assert np.array_equal(ids, want_ids) and np.array_equal(shared, want_shared), tau


def test_sharing_hand_worked_and_errors():
    masks = np.array([[1, 1, 0, 0, 0, 0], [1, 1, 1, 0, 0, 0], [1, 0, 1, 0, 0, 0], [1, 1, 0, 0, 0, 0]], np.uint8)
    ids, shared = pkg.share_timesteps(masks, 0.75)
    assert ids.tolist() == [0, 0, 1, 0] and shared.tolist() == [[1, 1, 1, 0, 0, 0], [1, 0, 1, 0, 0, 0]]
    lib = pkg.load_library()
    u8p, i32p = C.POINTER(C.c_uint8), C.POINTER(C.c_int32)
    cl, sh, n = np.zeros(4, np.int32), np.zeros_like(masks), C.c_int32(0)
    args = (masks.ctypes.data_as(u8p), 4, 6, 0.75, cl.ctypes.data_as(i32p), sh.ctypes.data_as(u8p), C.byref(n))
    assert lib.calibatt_share_timesteps(*args) == 0 and n.value == 2
    assert lib.calibatt_share_timesteps(None, *args[1:]) == -1
    assert lib.calibatt_share_timesteps(args[0], 0, *args[2:]) == -2
    assert lib.calibatt_share_timesteps(*args[:3], float("nan"), *args[4:]) == -2


def test_dictionary_masks_share_at_late_timesteps():
    """The time-coherent mask generator behind `bench.py --dictionary`: the kept fraction falls with the
    timestep, late timesteps resemble each other, and the library clusters them exactly as the oracle does."""
    from workloads import dictionary_head_masks

    masks = dictionary_head_masks(0, 3, steps=12, name="wan480")
    dens = masks.mean(axis=(1, 2))
    assert masks.shape[0] == 12 and masks.shape[1] == masks.shape[2] and (np.diff(dens) <= 1e-9).all()
    assert (masks[:, np.arange(masks.shape[1]), np.arange(masks.shape[1])] == 1).all()
    cluster, shared = pkg.share_timesteps(masks, 0.9)
    want_cluster, want_shared = sl.share_timesteps(masks.reshape(12, -1), 0.9)
    assert cluster.tolist() == list(want_cluster)
    assert (shared.reshape(len(want_shared), -1) == np.asarray(want_shared)).all()
    assert shared.shape[0] < 12  # something is shared
    assert sl.iou_skipped(masks[10].ravel(), masks[11].ravel()) > sl.iou_skipped(masks[0].ravel(), masks[1].ravel())
