"""Skip-list tools of the paper's supplement (Section A.2 "Skip-List Memory
Optimization", Section A.3 "Timestep Mask Sharing"), as plain Python/NumPy.

TEST INFRASTRUCTURE ONLY - never imported by the product package.

* A block-row of a mask is stored as its maximal runs of kept blocks
  ("intervals", [start, end) in key-block units).
* Interval merging: rows with more intervals than a target width get nearby
  intervals merged, i.e. the skipped blocks between them are marked as kept,
  until they fit.  The target is a percentile of the interval counts of all
  rows handed in (one layer in the paper).  The paper does not say which
  intervals merge first or how the percentile is taken; readings: the smallest
  gap first, the leftmost among equal gaps; nearest-rank percentile (the
  smallest count w such that at least pct percent of the rows have <= w).
* Timestep sharing, per (layer, head): timesteps are visited in ascending
  order; a timestep joins the first cluster (in order of creation) in which its
  IoU of *skipped*-block sets with every member is at least tau, else it
  founds a new cluster; a cluster's mask is the OR of its members' kept
  blocks.  Two masks that skip nothing have IoU 1.
* Flat ("1D") layout: all intervals of all rows in one array plus one offset
  per row.  The packed word used by the library holds the interval's start in
  its low 16 bits and the number of kept blocks before it in the row in its
  high 16 bits; a row of n intervals has n + 1 words, the last one carrying
  (0, total kept blocks).
"""
from __future__ import annotations

import math
from typing import List, Tuple

import numpy as np


def row_intervals(row) -> List[Tuple[int, int]]:
    """Maximal runs of non-zero entries as [start, end) pairs."""
    out = []
    start = None
    for c, x in enumerate(list(row) + [0]):
        if x and start is None:
            start = c
        elif not x and start is not None:
            out.append((start, c))
            start = None
    return out


def merge_row(row, max_intervals: int) -> np.ndarray:
    """Fill the smallest gaps (leftmost first among equals) until the row has at
    most ``max_intervals`` intervals (at least 1 is always allowed)."""
    r = (np.asarray(row) != 0).astype(np.uint8)
    limit = max(int(max_intervals), 1)
    while True:
        iv = row_intervals(r)
        if len(iv) <= limit:
            return r
        gaps = [(iv[i + 1][0] - iv[i][1], i) for i in range(len(iv) - 1)]
        _, i = min(gaps)
        r[iv[i][1] : iv[i + 1][0]] = 1


def interval_counts(mask: np.ndarray) -> np.ndarray:
    m = np.asarray(mask)
    flat = m.reshape(-1, m.shape[-1])
    return np.array([len(row_intervals(r)) for r in flat], dtype=np.int64).reshape(m.shape[:-1])


def percentile_width(counts, pct: float) -> int:
    """Nearest-rank percentile of the interval counts."""
    c = sorted(int(x) for x in np.asarray(counts).reshape(-1))
    if not c:
        return 0
    rank = max(1, math.ceil(pct / 100.0 * len(c)))
    return c[min(rank, len(c)) - 1]


def merge_mask(mask: np.ndarray, pct: float) -> Tuple[np.ndarray, int]:
    """Merge every row of ``mask[..., nbk]`` down to the pct-th percentile of the
    rows' interval counts.  Returns (merged uint8 mask, width)."""
    m = (np.asarray(mask) != 0).astype(np.uint8)
    width = percentile_width(interval_counts(m), pct)
    flat = m.reshape(-1, m.shape[-1]).copy()
    for i in range(flat.shape[0]):
        flat[i] = merge_row(flat[i], width)
    return flat.reshape(m.shape), width


def iou_skipped(a, b) -> float:
    sa, sb = np.asarray(a) == 0, np.asarray(b) == 0
    union = int((sa | sb).sum())
    return 1.0 if union == 0 else int((sa & sb).sum()) / union


def share_timesteps(masks: np.ndarray, tau: float) -> Tuple[np.ndarray, np.ndarray]:
    """masks[T, ...] of one (layer, head) -> (cluster id per timestep, shared
    masks [n_clusters, ...])."""
    m = (np.asarray(masks) != 0).astype(np.uint8)
    clusters: List[List[int]] = []
    ids = np.zeros(m.shape[0], dtype=np.int32)
    for t in range(m.shape[0]):
        for ci, members in enumerate(clusters):
            if all(iou_skipped(m[t], m[u]) >= tau for u in members):
                members.append(t)
                ids[t] = ci
                break
        else:
            clusters.append([t])
            ids[t] = len(clusters) - 1
    shared = np.stack([np.bitwise_or.reduce(m[members], axis=0) for members in clusters])
    return ids, shared


def encode_intervals(mask_rows: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Flat layout of the rows of ``mask_rows[n_rows, nbk]``: (iv_ptr int32
    [n_rows + 1], words uint32) with one terminating word per row."""
    m = np.asarray(mask_rows)
    ptr = [0]
    words: List[int] = []
    for r in range(m.shape[0]):
        before = 0
        for (s, e) in row_intervals(m[r]):
            words.append(s | (before << 16))
            before += e - s
        words.append(before << 16)
        ptr.append(len(words))
    return np.array(ptr, dtype=np.int32), np.array(words, dtype=np.uint32)


def decode_intervals(iv_ptr, words, nbk: int) -> np.ndarray:
    """Inverse of ``encode_intervals``."""
    n_rows = len(iv_ptr) - 1
    out = np.zeros((n_rows, nbk), dtype=np.uint8)
    for r in range(n_rows):
        w = [int(x) for x in words[iv_ptr[r] : iv_ptr[r + 1]]]
        for i in range(len(w) - 1):
            start, before = w[i] & 0xFFFF, w[i] >> 16
            length = (w[i + 1] >> 16) - before
            out[r, start : start + length] = 1
    return out


def bytes_2d(n_masks: int, n_blocks: int, width: int, bytes_per_entry: int = 2) -> int:
    """Footprint of the padded 2D layout: per mask n_blocks rows of ``width``
    entries plus one count column."""
    return n_masks * n_blocks * (width + 1) * bytes_per_entry
