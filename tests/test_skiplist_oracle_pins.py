"""Pins for the skip-list tools (CPU only): interval runs, merging, percentile
width, timestep sharing, flat interval layout, footprint arithmetic."""
import itertools

import numpy as np
import pytest

from oracle import skiplist as sl


def test_intervals_hand_worked():
    assert sl.row_intervals([1, 1, 0, 0, 1, 0, 1, 1, 1]) == [(0, 2), (4, 5), (6, 9)]
    assert sl.row_intervals([0, 0, 0]) == []
    assert sl.row_intervals([3]) == [(0, 1)]
    assert sl.row_intervals([0, 1, 0]) == [(1, 2)]
    # alternating pattern: ceil(n/2) intervals, the worst case of the supplement (N_B / 2)
    assert len(sl.row_intervals([1, 0] * 295 + [1])) == 296


def test_merge_hand_worked():
    row = [1, 0, 0, 1, 0, 1, 1, 0, 0, 0, 1]       # intervals (0,1) (3,4) (5,7) (10,11); gaps 2, 1, 3
    assert sl.merge_row(row, 4).tolist() == row
    assert sl.merge_row(row, 3).tolist() == [1, 0, 0, 1, 1, 1, 1, 0, 0, 0, 1]   # gap of 1 filled
    assert sl.merge_row(row, 2).tolist() == [1, 1, 1, 1, 1, 1, 1, 0, 0, 0, 1]   # then the gap of 2
    assert sl.merge_row(row, 1).tolist() == [1] * 11
    assert sl.merge_row(row, 0).tolist() == [1] * 11                             # at least one interval
    assert sl.merge_row([1, 0, 1, 0, 1], 2).tolist() == [1, 1, 1, 0, 1]          # equal gaps: leftmost first
    assert sl.merge_row([0, 0, 0], 1).tolist() == [0, 0, 0]


@pytest.mark.parametrize("seed", range(20))
def test_merge_is_a_cheapest_superset(seed):
    """Exhaustive check on short rows: the merged row is a superset with at most
    w intervals, and no superset with at most w intervals adds fewer blocks."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(3, 11))
    row = (rng.random(n) < 0.5).astype(np.uint8)
    w = int(rng.integers(1, 4))
    merged = sl.merge_row(row, w)
    assert (merged >= row).all() and len(sl.row_intervals(merged)) <= max(w, 1)
    zeros = np.flatnonzero(row == 0)
    best = None
    for k in range(len(zeros) + 1):
        for add in itertools.combinations(zeros, k):
            cand = row.copy()
            cand[list(add)] = 1
            if len(sl.row_intervals(cand)) <= w:
                best = k
                break
        if best is not None:
            break
    assert int(merged.sum() - row.sum()) == best


def test_percentile_width_nearest_rank():
    counts = [1, 2, 3, 4, 5, 6, 7, 8, 9, 10]
    assert sl.percentile_width(counts, 100) == 10
    assert sl.percentile_width(counts, 90) == 9
    assert sl.percentile_width(counts, 95) == 10
    assert sl.percentile_width(counts, 50) == 5
    assert sl.percentile_width(counts, 1) == 1
    assert sl.percentile_width([7], 90) == 7
    assert sl.percentile_width([], 90) == 0
    many = [3] * 95 + [50] * 5
    assert sl.percentile_width(many, 95) == 3 and sl.percentile_width(many, 96) == 50


def test_merge_mask_only_touches_outlier_rows():
    rng = np.random.default_rng(3)
    m = (rng.random((2, 20, 30)) < 0.4).astype(np.uint8)
    merged, width = sl.merge_mask(m, 90)
    counts = sl.interval_counts(m)
    assert width == sl.percentile_width(counts, 90)
    assert (sl.interval_counts(merged) <= width).all()
    untouched = counts <= width
    assert (merged[untouched] == m[untouched]).all()
    assert (merged >= m).all()
    same, w100 = sl.merge_mask(m, 100)
    assert (same == m).all() and w100 == counts.max()


def test_iou_hand_worked():
    a = np.array([1, 1, 0, 0, 0, 1])
    b = np.array([1, 0, 0, 0, 1, 1])
    assert sl.iou_skipped(a, b) == 2 / 4      # skipped {2,3,4} and {1,2,3}
    assert sl.iou_skipped(a, a) == 1.0
    assert sl.iou_skipped(np.ones(4), np.ones(4)) == 1.0
    assert sl.iou_skipped(np.ones(4), np.array([1, 1, 1, 0])) == 0.0


def test_sharing_hand_worked():
    t0 = [1, 1, 0, 0, 0, 0]
    t1 = [1, 1, 1, 0, 0, 0]   # IoU(t0, t1) = 3/4
    t2 = [1, 0, 1, 0, 0, 0]   # IoU(t0, t2) = 3/5, IoU(t1, t2) = 3/4
    t3 = [1, 1, 0, 0, 0, 0]   # = t0
    masks = np.array([t0, t1, t2, t3], np.uint8)
    ids, shared = sl.share_timesteps(masks, 0.75)
    # t1 joins t0; t2 fails against t0 (0.6) -> new cluster; t3 joins the first cluster (IoU 1 and 0.75)
    assert ids.tolist() == [0, 0, 1, 0]
    assert shared.tolist() == [[1, 1, 1, 0, 0, 0], [1, 0, 1, 0, 0, 0]]
    ids, shared = sl.share_timesteps(masks, 0.76)
    assert ids.tolist() == [0, 1, 2, 0]
    ids, shared = sl.share_timesteps(masks, 0.0)
    assert ids.tolist() == [0, 0, 0, 0] and shared.tolist() == [[1, 1, 1, 0, 0, 0]]
    ids, shared = sl.share_timesteps(masks, 1.0)
    assert ids.tolist() == [0, 1, 2, 0] and (shared[0] == masks[0]).all()


def test_sharing_invariants():
    rng = np.random.default_rng(4)
    base = (rng.random((6, 12)) < 0.4).astype(np.uint8)
    masks = np.stack([np.where(rng.random(base.shape) < 0.03 * t, 1 - base, base) for t in range(10)])
    for tau in (0.5, 0.8, 0.95):
        ids, shared = sl.share_timesteps(masks, tau)
        assert ids[0] == 0 and shared.shape[0] == ids.max() + 1
        for c in range(shared.shape[0]):
            members = np.flatnonzero(ids == c)
            assert (shared[c] == masks[members].max(axis=0)).all()     # OR of kept blocks
            for a, b in itertools.combinations(members, 2):            # cliques: every pair passes
                assert sl.iou_skipped(masks[a], masks[b]) >= tau
        # a shared mask never skips a block one of its members keeps
        assert all((shared[ids[t]] >= masks[t]).all() for t in range(10))


def test_flat_layout_hand_worked_and_round_trip():
    m = np.array([[1, 1, 0, 0, 1, 0, 1, 1, 1], [0] * 9, [1] * 9], np.uint8)
    ptr, words = sl.encode_intervals(m)
    assert ptr.tolist() == [0, 4, 5, 7]
    assert words.tolist() == [0 | (0 << 16), 4 | (2 << 16), 6 | (3 << 16), 6 << 16, 0, 0, 9 << 16]
    assert (sl.decode_intervals(ptr, words, 9) == m).all()
    rng = np.random.default_rng(5)
    big = (rng.random((50, 300)) < 0.3).astype(np.uint8)
    ptr, words = sl.encode_intervals(big)
    assert (sl.decode_intervals(ptr, words, 300) == big).all()
    assert len(words) == sl.interval_counts(big).sum() + 50


def test_footprint_of_the_untrimmed_2d_layout_matches_the_paper():
    # supplement A.2: 52 GB for Wan 14B at 720p = 50 steps x 40 layers x 40 heads masks of 591 rows,
    # full width 591 (start/end entries of up to 295 intervals) plus the count column, 2 bytes each
    b = sl.bytes_2d(50 * 40 * 40, 591, 591)
    assert round(b / 2 ** 30) == 52
