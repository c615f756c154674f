"""Pins for the pattern-compilation oracle (CPU only): a hand-worked example,
an independent NumPy construction, structural invariants and the error rules."""
import json
import os

import numpy as np
import pytest

from oracle import PatternError, compile_pattern, pattern_sizes
from workloads import random_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load_worked_example():
    with open(os.path.join(GOLDEN, "pattern_worked_example.json")) as f:
        return json.load(f)


def check_against_worked_example(compile_fn):
    ex = load_worked_example()
    mask = np.array(ex["mask"], dtype=np.uint8)
    repeat = np.array(ex["repeat"], dtype=np.int32)
    for order in (0, 1, 2, 3, 4):
        p = compile_fn(mask, repeat, ex["H"], ex["N"], ex["block_q"], ex["block_k"], order)
        assert (p["nnz"], p["n_work"], p["n_repeat"]) == (ex["nnz"], ex["n_work"], ex["n_repeat"])
        for name in ("row_ptr", "col_idx", "repeat_src"):
            assert p[name].tolist() == ex[name], (order, name)
        for name in ("work", "fan_ptr", "fan_dst"):
            assert p[name].tolist() == ex[f"order{order}"][name], (order, name)
        if order >= 3:  # the groups of the XCD-aware orders
            assert np.asarray(p["group_ptr"]).tolist() == ex[f"order{order}"]["group_ptr"], order


def independent_numpy_compile(mask, repeat, H, N, bq, bk, order):
    """Second construction with library primitives (flatnonzero, cumsum,
    lexsort) instead of loops."""
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask = np.asarray(mask).reshape(H, nbq, nbk) != 0
    rep = np.full((H, nbq), -1, np.int64) if repeat is None else np.asarray(repeat, np.int64).reshape(H, nbq)
    live = rep < 0
    counts = np.where(live, mask.sum(axis=2), 0).reshape(-1)
    row_ptr = np.concatenate([[0], np.cumsum(counts)])
    eff = mask & live[:, :, None]
    col_idx = np.nonzero(eff.reshape(H * nbq, nbk))[1]
    ids = np.flatnonzero(live.reshape(-1))
    hh, rr = ids // nbq, ids % nbq
    group_ptr = None
    if order == 0:
        perm = np.arange(ids.size)
    elif order == 1:
        perm = np.lexsort((rr, hh, -counts[ids]))
    elif order == 2:
        perm = np.lexsort((rr, -counts[ids], hh))
    else:
        # deal heads (heaviest first) to the lightest of 8 groups, with a heap
        import heapq

        weight = np.array([counts[h * nbq : (h + 1) * nbq].sum() for h in range(H)])
        heap = [(0, g) for g in range(8)]
        group_of = np.zeros(H, np.int64)
        rank_in_group = np.zeros(H, np.int64)
        size = [0] * 8
        for h in np.lexsort((np.arange(H), -weight)):
            load, g = heapq.heappop(heap)
            group_of[h], rank_in_group[h] = g, size[g]
            size[g] += 1
            heapq.heappush(heap, (load + int(weight[h]), g))
        c_live = counts[ids]
        long_ = 2 * c_live * ids.size > 3 * c_live.sum()
        if order == 3:
            # one lexsort: group, long rows before the others, then (count desc for long rows), head rank, r
            perm = np.lexsort((rr, rank_in_group[hh], np.where(long_, -c_live, 0), ~long_, group_of[hh]))
        else:
            # order 4: group, head rank, count descending, r
            perm = np.lexsort((rr, -c_live, rank_in_group[hh], group_of[hh]))
        group_ptr = np.concatenate([[0], np.cumsum(np.bincount(group_of[hh], minlength=8))])
    work = ids[perm]
    fan = [np.flatnonzero(rep[w // nbq] == w % nbq) for w in work]
    fan_ptr = np.concatenate([[0], np.cumsum([len(f) for f in fan])])
    fan_dst = np.concatenate(fan) if fan else np.zeros(0, np.int64)
    out = dict(row_ptr=row_ptr, col_idx=col_idx, repeat_src=rep.reshape(-1), work=work, fan_ptr=fan_ptr, fan_dst=fan_dst)
    if group_ptr is not None:
        out["group_ptr"] = group_ptr
    return out


def check_invariants(p, mask, repeat, H, N, bq, bk, order):
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask = np.asarray(mask).reshape(H, nbq, nbk) != 0
    rep = np.full((H, nbq), -1, np.int64) if repeat is None else np.asarray(repeat, np.int64).reshape(H, nbq)
    row_ptr, col_idx, work = p["row_ptr"], p["col_idx"], p["work"]
    assert row_ptr[0] == 0 and row_ptr[-1] == p["nnz"] == col_idx.size
    assert (np.diff(row_ptr) >= 0).all()
    # round trip on non-repeated rows; repeated rows are empty
    back = np.zeros((H * nbq, nbk), dtype=bool)
    for i in range(H * nbq):
        cols = col_idx[row_ptr[i] : row_ptr[i + 1]]
        assert (np.diff(cols) > 0).all()
        back[i, cols] = True
    live = (rep < 0).reshape(-1)
    assert (back[live] == mask.reshape(H * nbq, nbk)[live]).all()
    assert not back[~live].any()
    # work is a permutation of the live ids; fan-out lists partition the repeated ones
    assert sorted(work.tolist()) == np.flatnonzero(live).tolist()
    assert p["n_work"] + p["n_repeat"] == H * nbq
    seen = []
    for i, w in enumerate(work):
        h, r = divmod(int(w), nbq)
        dst = p["fan_dst"][p["fan_ptr"][i] : p["fan_ptr"][i + 1]]
        assert (np.diff(dst) > 0).all()
        assert (rep[h, dst] == r).all()
        seen += [h * nbq + int(d) for d in dst]
    assert sorted(seen) == np.flatnonzero(~live).tolist()
    cnt = np.diff(row_ptr)[work]
    if order == 1:
        assert (np.diff(cnt) <= 0).all()
    if order == 2:
        assert (np.diff(work // nbq) >= 0).all()
    if order in (3, 4):
        gp = p["group_ptr"]
        assert p["n_groups"] == 8 and gp[0] == 0 and gp[8] == p["n_work"] and (np.diff(gp) >= 0).all()
        heads_of = [sorted(set((work[gp[g] : gp[g + 1]] // nbq).tolist())) for g in range(8)]
        assert sorted(h for hs in heads_of for h in hs) == sorted(set((work // nbq).tolist()))  # a head lives in one group
        for g in range(8):
            seg = work[gp[g] : gp[g + 1]]
            hs = seg // nbq
            c_seg = cnt[gp[g] : gp[g + 1]]
            if order == 3:
                # long rows lead, longest first; after them a head's rows are contiguous and ascending
                is_long = 2 * c_seg * p["n_work"] > 3 * p["nnz"]
                n_long = int(is_long.sum())
                assert is_long[:n_long].all() and (np.diff(c_seg[:n_long]) <= 0).all()
                for h in set(hs[n_long:].tolist()):
                    idx = np.flatnonzero(hs[n_long:] == h)
                    assert (np.diff(idx) == 1).all() and (np.diff(seg[n_long:][idx]) > 0).all()
            else:
                # a head's rows are contiguous, longest first, r ascending among equal counts
                for h in set(hs.tolist()):
                    idx = np.flatnonzero(hs == h)
                    assert (np.diff(idx) == 1).all()
                    c_h, r_h = c_seg[idx], seg[idx]
                    assert (np.diff(c_h) <= 0).all() and (np.diff(r_h)[np.diff(c_h) == 0] > 0).all()
        # greedy dealing keeps the groups within one head's weight of each other
        w = np.array([cnt[gp[g] : gp[g + 1]].sum() for g in range(8)])
        per_head = {}
        for x, c in zip(work, cnt):
            per_head[x // nbq] = per_head.get(x // nbq, 0) + c
        if len(per_head) >= 8:
            assert w.max() - w.min() <= max(per_head.values())
    else:
        assert p["n_groups"] == 1 and p["group_ptr"][0] == 0 and p["group_ptr"][1] == p["n_work"]


def test_oracle_worked_example():
    check_against_worked_example(compile_pattern)


@pytest.mark.parametrize("seed", range(40))
def test_oracle_vs_independent_construction(seed):
    rng = np.random.default_rng(seed)
    H = int(rng.integers(1, 4))
    bq, bk = int(rng.choice([4, 8, 16])), int(rng.choice([4, 8, 16]))
    N = int(rng.integers(1, 200))
    nbq, nbk = -(-N // bq), -(-N // bk)
    dens = float(rng.choice([0.0, 0.1, 0.5, 0.9, 1.0]))
    mask, repeat = random_mask(seed, H, nbq, nbk, dens, float(rng.choice([0, 0.2, 0.6])), tail_partial=(N % bq) != 0)
    mask = mask * rng.integers(1, 255, size=mask.shape).astype(np.uint8)  # any non-zero byte = kept
    for order in (0, 1, 2, 3, 4):
        p = compile_pattern(mask, repeat, H, N, bq, bk, order)
        q = independent_numpy_compile(mask, repeat, H, N, bq, bk, order)
        for name in q:
            assert p[name].tolist() == np.asarray(q[name]).tolist(), (order, name)
        check_invariants(p, mask, repeat, H, N, bq, bk, order)
        assert pattern_sizes(mask, repeat, H, N, bq, bk) == (p["nnz"], p["n_work"], p["n_repeat"])


def test_oracle_no_repeat_argument():
    mask, _ = random_mask(3, 2, 6, 6, 0.5)
    a = compile_pattern(mask, None, 2, 48, 8, 8, 1)
    b = compile_pattern(mask, np.full((2, 6), -1, np.int32), 2, 48, 8, 8, 1)
    for name in ("row_ptr", "col_idx", "repeat_src", "work", "fan_ptr", "fan_dst"):
        assert a[name].tolist() == b[name].tolist()
    assert a["n_repeat"] == 0 and a["fan_dst"].size == 0


REJECTED = [
    # repeat row (H=1, nbq=4), N, block_q, expected kind
    ([-1, 4, -1, -1], 32, 8, "range"),
    ([-1, -2, -1, -1], 32, 8, "range"),
    ([-1, 1, -1, -1], 32, 8, "range"),  # repeats itself
    ([-1, 0, 1, -1], 32, 8, "chain"),
    ([1, 0, -1, -1], 32, 8, "chain"),
    ([3, -1, -1, -1], 30, 8, "tail"),  # source is the 6-row last block, destination is full
]


def rejected_cases():
    return REJECTED


@pytest.mark.parametrize("rep,N,bq,kind", REJECTED)
def test_oracle_rejects(rep, N, bq, kind):
    mask = np.ones((1, 4, 4), dtype=np.uint8)
    with pytest.raises(PatternError) as e:
        compile_pattern(mask, np.array([rep], np.int32), 1, N, bq, 8, 1)
    assert e.value.kind == kind


def test_oracle_accepts_short_destination():
    mask = np.ones((1, 4, 4), dtype=np.uint8)
    p = compile_pattern(mask, np.array([[-1, -1, -1, 0]], np.int32), 1, 30, 8, 8, 0)
    assert p["fan_dst"].tolist() == [3] and p["n_work"] == 3
