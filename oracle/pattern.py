"""Integer oracle for pattern compilation: block mask + repeat map -> index lists.

TEST INFRASTRUCTURE ONLY - never imported by the product package.

The paper (Section 3.4; supplement Section A.2) turns every calibrated block
mask into a read-only per-query-block-row list of the key block-columns to
compute, built once and kept on the GPU.  The form fixed for this library is a
padding-free list of block *indices* (the supplement's "1D" idea taken down to
single blocks): for each non-repeated query block the ascending kept columns.
Repetition (Section 3.3) is a per-head map query block -> source query block.

Outputs, all int32, all uniquely determined by the inputs:

row_ptr[H*nbq + 1]  exclusive prefix sum, in (h, r) order, of the kept count of
                    each query block; a repeated block counts 0 whatever its
                    mask row says.
col_idx[nnz]        ascending kept columns of each non-repeated block.
repeat_src[H*nbq]   -1, or the source block (same head).
work[n_work]        ids h*nbq + r of the non-repeated blocks in schedule order:
                    order 0: (h, r) ascending;
                    order 1: kept count descending, then h, then r;
                    order 2: h ascending, then kept count descending, then r;
                    order 3: heads are dealt to N_GROUPS = 8 groups (one per
                             XCD of the target GPU): heads sorted by total kept
                             blocks descending (then h), each given to the group
                             with the smallest load so far (then lowest group);
                             a group's segment of work first lists its "long"
                             blocks (kept count > 1.5 x the mean over all
                             computed blocks, i.e. 2*count*n_work > 3*nnz) by
                             count descending, then dealing order of the head,
                             then r; after them the remaining blocks head by
                             head in dealing order, r ascending.  Group 0's
                             segment comes first, then group 1, ...
                    order 4: groups as for order 3; a group's segment lists
                             its heads in dealing order and, within a head, the
                             blocks by count descending, then r.
group_ptr[9]        orders 3, 4: start of each group's segment in work, last
                    entry n_work.  Other orders: one group, [0, n_work, ...].
fan_ptr[n_work+1], fan_dst[n_repeat]
                    for work item i the ascending list of blocks r' of the same
                    head with repeat[h, r'] == r.

Rejected inputs (exceptions here, status codes in the library):
 range : repeat value outside {-1} U [0, nbq), or a block repeating itself
 chain : the source of a repeated block is itself repeated
 tail  : the source is the shorter last block but the destination is a full one
"""
from __future__ import annotations

import numpy as np


N_GROUPS = 8


class PatternError(ValueError):
    def __init__(self, kind: str, msg: str = ""):
        super().__init__(f"{kind}: {msg}")
        self.kind = kind


def _dims(H, N, block_q, block_k):
    if H <= 0 or N <= 0 or block_q <= 0 or block_k <= 0:
        raise PatternError("shape", "non-positive dimension")
    return -(-N // block_q), -(-N // block_k)


def _check_repeat(rep, H, nbq, N, block_q):
    last_partial = (N % block_q) != 0
    for h in range(H):
        for r in range(nbq):
            s = int(rep[h, r])
            if s == -1:
                continue
            if s < -1 or s >= nbq or s == r:
                raise PatternError("range", f"repeat[{h},{r}]={s}")
            if rep[h, s] != -1:
                raise PatternError("chain", f"repeat[{h},{r}]={s} which repeats {int(rep[h, s])}")
            if last_partial and s == nbq - 1 and r != nbq - 1:
                raise PatternError("tail", f"repeat[{h},{r}] is the short last block")


def pattern_sizes(mask, repeat, H, N, block_q, block_k):
    """(nnz, n_work, n_repeat) after validation."""
    nbq, nbk = _dims(H, N, block_q, block_k)
    mask = np.asarray(mask).reshape(H, nbq, nbk)
    rep = np.full((H, nbq), -1, dtype=np.int64) if repeat is None else np.asarray(repeat, dtype=np.int64).reshape(H, nbq)
    _check_repeat(rep, H, nbq, N, block_q)
    nnz = 0
    n_rep = 0
    for h in range(H):
        for r in range(nbq):
            if rep[h, r] >= 0:
                n_rep += 1
            else:
                nnz += int(np.count_nonzero(mask[h, r]))
    return nnz, H * nbq - n_rep, n_rep


def compile_pattern(mask, repeat, H, N, block_q, block_k, order=1):
    """Returns a dict of int32 arrays: row_ptr, col_idx, repeat_src, work,
    fan_ptr, fan_dst, plus ints nbq, nbk, nnz, n_work, n_repeat."""
    nbq, nbk = _dims(H, N, block_q, block_k)
    if order not in (0, 1, 2, 3, 4):
        raise PatternError("unsupported", f"order={order}")
    mask = np.asarray(mask).reshape(H, nbq, nbk)
    rep = np.full((H, nbq), -1, dtype=np.int64) if repeat is None else np.asarray(repeat, dtype=np.int64).reshape(H, nbq)
    _check_repeat(rep, H, nbq, N, block_q)

    row_ptr = [0]
    col_idx = []
    counts = {}
    for h in range(H):
        for r in range(nbq):
            cols = [] if rep[h, r] >= 0 else [c for c in range(nbk) if mask[h, r, c] != 0]
            col_idx.extend(cols)
            row_ptr.append(len(col_idx))
            counts[(h, r)] = len(cols)

    items = [(h, r) for h in range(H) for r in range(nbq) if rep[h, r] < 0]
    if order == 1:
        items.sort(key=lambda hr: (-counts[hr], hr[0], hr[1]))
    elif order == 2:
        items.sort(key=lambda hr: (hr[0], -counts[hr], hr[1]))
    group_ptr = [0] + [len(items)] * N_GROUPS
    if order in (3, 4):
        weight = [sum(counts[(h, r)] for r in range(nbq)) for h in range(H)]
        load = [0] * N_GROUPS
        members = [[] for _ in range(N_GROUPS)]
        for h in sorted(range(H), key=lambda h: (-weight[h], h)):
            g = min(range(N_GROUPS), key=lambda g: (load[g], g))
            members[g].append(h)
            load[g] += weight[h]
        items = []
        group_ptr = [0]
        nnz_total, n_live = len(col_idx), sum(1 for h in range(H) for r in range(nbq) if rep[h, r] < 0)
        is_long = lambda hr: 2 * counts[hr] * n_live > 3 * nnz_total
        for g in range(N_GROUPS):
            live = [(h, r) for h in members[g] for r in range(nbq) if rep[h, r] < 0]
            rank = {h: i for i, h in enumerate(members[g])}
            if order == 3:
                items.extend(sorted((hr for hr in live if is_long(hr)), key=lambda hr: (-counts[hr], rank[hr[0]], hr[1])))
                items.extend(hr for hr in live if not is_long(hr))
            else:
                for h in members[g]:
                    items.extend(sorted((hr for hr in live if hr[0] == h), key=lambda hr: (-counts[hr], hr[1])))
            group_ptr.append(len(items))
    work = [h * nbq + r for (h, r) in items]

    fan_ptr = [0]
    fan_dst = []
    for (h, r) in items:
        fan_dst.extend(r2 for r2 in range(nbq) if rep[h, r2] == r)
        fan_ptr.append(len(fan_dst))

    i32 = lambda a: np.asarray(a, dtype=np.int32).reshape(-1)
    return dict(
        nbq=nbq, nbk=nbk, nnz=len(col_idx), n_work=len(work), n_repeat=len(fan_dst),
        row_ptr=i32(row_ptr), col_idx=i32(col_idx), repeat_src=i32(rep),
        work=i32(work), fan_ptr=i32(fan_ptr), fan_dst=i32(fan_dst),
        n_groups=N_GROUPS if order in (3, 4) else 1, group_ptr=i32(group_ptr),
    )
