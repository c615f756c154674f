"""fp64 definition of masked ("restricted") softmax attention.

TEST INFRASTRUCTURE ONLY - never imported by the product package.

What is computed (paper, Section 2, Eq. 1-2; Section 3.2 for the meaning of the
block mask; Section 3.3/3.4 for repetition):

* Queries, keys and values of one head are split into contiguous blocks of
  ``block_q`` / ``block_k`` tokens (the index sets I_r, J_c of Eq. 3).
* A query in block r attends only to keys j < N whose block c = j // block_k has
  mask[h, r, c] != 0.  Skipped blocks contribute exactly zero probability,
  which is written here as a logit of -inf before the softmax of Eq. 1.
* A = P V (Eq. 2) over the surviving keys.  A query with no surviving key gets
  an all-zero output (reading chosen for the case the paper does not cover).
* A query block r with repeat[h, r] = s >= 0 is not computed: its rows are a
  plain copy of the rows of block s of the same head (the block-level form of
  "compute anchors, broadcast the result", Section 3.3).

There is no tiling, no online softmax and no reordering: the logits of a whole
query block against *all* N keys are materialised, masked, and pushed through a
max-subtracted softmax, exactly as the definition reads.
"""
from __future__ import annotations

from typing import Iterable, List, Sequence, Tuple

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    u32 = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u32.view(np.float32).astype(np.float64)


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of IEEE binary16 bit patterns (uint16) to fp64, field by field."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.int64)
    sign = np.where(b >> 15, -1.0, 1.0)
    exp = (b >> 10) & 0x1F
    frac = (b & 0x3FF).astype(np.float64)
    normal = (1.0 + frac / 1024.0) * np.exp2((exp - 15).astype(np.float64))
    subnormal = (frac / 1024.0) * 2.0 ** -14
    special = np.where(frac == 0, np.inf, np.nan)
    return sign * np.where(exp == 0, subnormal, np.where(exp == 31, special, normal))


def _to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f64(bits)
    if dtype == "f16":
        return f16_bits_to_f64(bits)
    raise ValueError(dtype)


def expand_block_mask(mask_row: np.ndarray, block_k: int, n_keys: int) -> np.ndarray:
    """Per-key boolean for one query block: key j is visible iff its block
    j // block_k is kept (Section 3.2: entry 1 = computed, 0 = skipped)."""
    j = np.arange(n_keys)
    return np.asarray(mask_row)[j // block_k] != 0


def restricted_softmax_rows(logits: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """Row softmax (Eq. 1) with invisible keys at -inf.  Rows with no visible
    key come back as all zeros."""
    s = np.where(visible[None, :], logits, -np.inf)
    if not visible.any():
        return np.zeros_like(s)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=1, keepdims=True)


def _block_output(qf, kf, vf, mask_row, r, scale, block_q, block_k, n):
    rows = slice(r * block_q, min((r + 1) * block_q, n))
    visible = expand_block_mask(mask_row, block_k, n)
    logits = scale * (qf[rows] @ kf.T)
    p = restricted_softmax_rows(logits, visible)
    return p @ vf, p


def sparse_attention(
    q_bits: np.ndarray,
    k_bits: np.ndarray,
    v_bits: np.ndarray,
    mask: np.ndarray,
    repeat,
    scale: float,
    block_q: int,
    block_k: int,
    return_probs: bool = False,
    dtype: str = "bf16",
):
    """Full output, fp64 [B, H, N, D].

    q/k/v: uint16 bf16 bits [B, H, N, D].  mask: [H, ceil(N/block_q),
    ceil(N/block_k)], non-zero = kept.  repeat: [H, ceil(N/block_q)] with -1 or
    the source query block, or None.  The same mask serves every batch index
    (the paper applies one calibrated mask to both guidance branches,
    supplement Section A).  With ``return_probs`` also returns P [B,H,N,N]
    (rows of repeated blocks left at zero) - small inputs only.
    """
    B, H, N, D = q_bits.shape
    nbq = -(-N // block_q)
    nbk = -(-N // block_k)
    mask = np.asarray(mask)
    assert mask.shape == (H, nbq, nbk), (mask.shape, (H, nbq, nbk))
    rep = np.full((H, nbq), -1, dtype=np.int64) if repeat is None else np.asarray(repeat, dtype=np.int64)
    out = np.zeros((B, H, N, D), dtype=np.float64)
    probs = np.zeros((B, H, N, N), dtype=np.float64) if return_probs else None
    for b in range(B):
        for h in range(H):
            qf = _to_f64(q_bits[b, h], dtype)
            kf = _to_f64(k_bits[b, h], dtype)
            vf = _to_f64(v_bits[b, h], dtype)
            for r in range(nbq):
                if rep[h, r] >= 0:
                    continue
                o, p = _block_output(qf, kf, vf, mask[h, r], r, scale, block_q, block_k, N)
                out[b, h, r * block_q : r * block_q + o.shape[0]] = o
                if return_probs:
                    probs[b, h, r * block_q : r * block_q + o.shape[0]] = p
            for r in range(nbq):
                s = int(rep[h, r])
                if s < 0:
                    continue
                n_rows = min((r + 1) * block_q, N) - r * block_q
                out[b, h, r * block_q : r * block_q + n_rows] = out[b, h, s * block_q : s * block_q + n_rows]
    if return_probs:
        return out, probs
    return out


def sparse_attention_blocks(
    q_bits: np.ndarray,
    k_bits: np.ndarray,
    v_bits: np.ndarray,
    mask: np.ndarray,
    repeat,
    scale: float,
    block_q: int,
    block_k: int,
    items: Iterable[Tuple[int, int, int]],
    dtype: str = "bf16",
) -> List[np.ndarray]:
    """Outputs of selected query blocks only: for each (b, h, r) in ``items`` an
    fp64 array [rows_in_block_r, D].  Same arithmetic as ``sparse_attention``;
    a repeated block returns the leading rows of its source block's output."""
    B, H, N, D = q_bits.shape
    nbq = -(-N // block_q)
    rep = np.full((H, nbq), -1, dtype=np.int64) if repeat is None else np.asarray(repeat, dtype=np.int64)
    mask = np.asarray(mask)
    results = []
    cache = {}
    for (b, h, r) in items:
        key = (b, h)
        if key not in cache:
            cache.clear()
            cache[key] = (
                _to_f64(q_bits[b, h], dtype),
                _to_f64(k_bits[b, h], dtype),
                _to_f64(v_bits[b, h], dtype),
            )
        qf, kf, vf = cache[key]
        n_rows = min((r + 1) * block_q, N) - r * block_q
        src = int(rep[h, r])
        rr = r if src < 0 else src
        o, _ = _block_output(qf, kf, vf, mask[h, rr], rr, scale, block_q, block_k, N)
        results.append(o[:n_rows].copy())
    return results


def sparse_attention_lse(q_bits, k_bits, mask, repeat, scale: float, block_q: int, block_k: int, dtype: str = "bf16") -> np.ndarray:
    """Per query the natural logarithm of the normaliser of Eq. 1 restricted to
    the kept keys: log sum_{j kept} exp(scale * q_i . k_j), fp64 [B, H, N]; -inf
    for a query that keeps no key; the rows of a repeated block carry the values
    of the leading rows of their source block."""
    B, H, N, D = q_bits.shape
    nbq = -(-N // block_q)
    rep = np.full((H, nbq), -1, dtype=np.int64) if repeat is None else np.asarray(repeat, dtype=np.int64)
    mask = np.asarray(mask)
    out = np.full((B, H, N), -np.inf, dtype=np.float64)
    for b in range(B):
        for h in range(H):
            qf, kf = _to_f64(q_bits[b, h], dtype), _to_f64(k_bits[b, h], dtype)
            for r in range(nbq):
                if rep[h, r] >= 0:
                    continue
                rows = slice(r * block_q, min((r + 1) * block_q, N))
                visible = expand_block_mask(mask[h, r], block_k, N)
                if not visible.any():
                    continue
                s = scale * (qf[rows] @ kf[visible].T)
                m = s.max(axis=1)
                out[b, h, rows] = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
            for r in range(nbq):
                src = int(rep[h, r])
                if src < 0:
                    continue
                n_rows = min((r + 1) * block_q, N) - r * block_q
                out[b, h, r * block_q : r * block_q + n_rows] = out[b, h, src * block_q : src * block_q + n_rows]
    return out
