"""The library's host-side anchor map (C ABI, no GPU) against the oracle's maps:
bit-exact index lists, error codes."""
import ctypes as C

import numpy as np
import pytest

import paper_2603_05503_amd as pkg
from oracle import anchor_token_maps


def _expected(N, F, Hs, Ws, k):
    q_index, src = anchor_token_maps(N, F, Hs, Ws, k)
    order = np.argsort(src, kind="stable")  # receivers grouped by computed query, ascending token
    counts = np.bincount(src, minlength=q_index.size)
    dst_ptr = np.concatenate([[0], np.cumsum(counts)])
    return q_index.astype(np.int32), dst_ptr.astype(np.int32), order.astype(np.int32)


CASES = [
    (14, 2, 3, 2, 1), (12, 2, 3, 2, 3), (6, 1, 6, 1, 2), (75, 3, 7, 3, 3), (420, 3, 7, 20, 2),
    (32760, 21, 30, 52, 5), (32760, 21, 30, 52, 1), (32760, 21, 30, 52, 30), (44520, 28, 30, 53, 5),
    (44776, 28, 30, 53, 7), (1, 1, 1, 1, 1), (9, 1, 1, 1, 1),
]


@pytest.mark.parametrize("N,F,Hs,Ws,k", CASES)
def test_map_matches_oracle(N, F, Hs, Ws, k):
    m = pkg.anchor_map(N, F, Hs, Ws, k)
    q_index, dst_ptr, dst_idx = _expected(N, F, Hs, Ws, k)
    assert m.n_q == q_index.size == F * k * Ws + N - F * Hs * Ws
    assert m.q_index.dtype == np.int32 and np.array_equal(m.q_index, q_index)
    assert np.array_equal(m.dst_ptr, dst_ptr)
    assert np.array_equal(m.dst_idx, dst_idx)
    assert np.array_equal(np.sort(m.dst_idx), np.arange(N))  # every token receives exactly once


def test_all_k_small_geometries():
    for Hs in range(1, 12):
        for k in range(1, Hs + 1):
            m = pkg.anchor_map(2 * Hs * 3 + 2, 2, Hs, 3, k)
            q_index, dst_ptr, dst_idx = _expected(2 * Hs * 3 + 2, 2, Hs, 3, k)
            assert np.array_equal(m.q_index, q_index) and np.array_equal(m.dst_ptr, dst_ptr)
            assert np.array_equal(m.dst_idx, dst_idx), (Hs, k)


@pytest.mark.parametrize("args", [(0, 1, 1, 1, 1), (10, 0, 1, 1, 1), (10, 1, 0, 1, 1), (10, 1, 1, 0, 1),
                                  (10, 1, 2, 2, 0), (10, 1, 2, 2, 3), (10, 3, 2, 2, 1), (-5, 1, 1, 1, 1)])
def test_shape_errors(args):
    with pytest.raises(pkg.CalibattError) as e:
        pkg.anchor_map(*args)
    assert e.value.status == -2


def test_null_count_pointer():
    lib = pkg.load_library()
    assert lib.calibatt_anchor_map(10, 1, 2, 2, 1, None, None, None, None) == -1


def test_size_query_writes_nothing():
    lib = pkg.load_library()
    n_q = C.c_int32(-1)
    buf = np.full(8, 77, np.int32)
    st = lib.calibatt_anchor_map(12, 2, 3, 2, 1, buf.ctypes.data_as(C.POINTER(C.c_int32)), None, None, C.byref(n_q))
    assert st == 0 and n_q.value == 4 and (buf == 77).all()


def test_attn_argument_errors_need_no_gpu():
    """Argument checks come before any HIP call."""
    lib = pkg.load_library()
    f = lib.calibatt_anchor_attn_fwd
    one = C.c_void_p(16)
    assert f(None, one, one, C.c_void_p(32), 1, 1, 8, 64, one, 1, one, one, one, 1, 1.0, None) == -1
    assert f(one, one, one, C.c_void_p(32), 1, 1, 8, 64, None, 1, one, one, one, 1, 1.0, None) == -1
    assert f(one, one, one, C.c_void_p(32), 0, 1, 8, 64, one, 1, one, one, one, 1, 1.0, None) == -2
    assert f(one, one, one, C.c_void_p(32), 1, 1, 8, 64, one, -1, one, one, one, 1, 1.0, None) == -2
    assert f(one, one, one, one, 1, 1, 8, 64, one, 1, one, one, one, 1, 1.0, None) == -2  # out aliases q
    assert f(one, one, one, C.c_void_p(32), 1, 1, 8, 96, one, 1, one, one, one, 1, 1.0, None) == -3
    assert f(one, one, one, C.c_void_p(32), 1, 1, 8, 64, None, 0, None, None, None, 0, 1.0, None) == 0  # no-op


@pytest.mark.parametrize("F,Hs,Ws,k", [(2, 3, 2, 1), (1, 6, 1, 2), (3, 7, 3, 3), (21, 30, 52, 5), (21, 30, 52, 1), (2, 9, 4, 9)])
def test_partner_matches_oracle(F, Hs, Ws, k):
    q_index, src = anchor_token_maps(F * Hs * Ws, F, Hs, Ws, k)
    got = pkg.anchor_partner(F, Hs, Ws, k)
    assert got.dtype == np.int32 and np.array_equal(got, q_index[src])


def test_partner_errors():
    lib = pkg.load_library()
    assert lib.calibatt_anchor_partner(1, 2, 2, 1, None) == -1
    buf = np.zeros(8, np.int32)
    p = buf.ctypes.data_as(C.POINTER(C.c_int32))
    assert lib.calibatt_anchor_partner(0, 2, 2, 1, p) == -2
    assert lib.calibatt_anchor_partner(1, 2, 2, 3, p) == -2
    one = C.c_void_p(16)
    f = lib.calibatt_spatial_similarity
    assert f(None, one, 1, 1, 8, 64, one, 8, 2, 1.0, one, one, None) == -1
    assert f(one, one, 1, 1, 8, 64, one, 9, 3, 1.0, one, one, None) == -2   # more tokens than N
    assert f(one, one, 1, 1, 8, 64, one, 8, 3, 1.0, one, one, None) == -2   # rows do not divide
    assert f(one, one, 1, 1, 8, 96, one, 8, 2, 1.0, one, one, None) == -3
