"""fp64 definitions of the calibration steps that produce a block mask (paper,
Section 3.2: Eq. 5 block energy, Eq. 6 smallest set of blocks reaching an energy
threshold, Eq. 7 threshold schedule, Eq. 8-9 cross-prompt vote; supplement
Section A.1 for the schedule parameters the paper uses).

TEST INFRASTRUCTURE ONLY - never imported by the product package.

Readings where the paper is silent:
* N not a multiple of the block: the last blocks are short; the energy of a
  short query block is averaged over the rows it has, so that every block-row
  still sums to 1 (the property the paper states for the 1/B average).
* Equal energies in the descending sort: the lower column index comes first.
* The running sum that is compared with the threshold is taken in fp64, in the
  sorted order, whatever the dtype of the energies handed in.
* A row whose total stays below the threshold (rounding) keeps every block.
"""
from __future__ import annotations

import math

import numpy as np

from .attention import bf16_bits_to_f64


def _energy_of_rows(q_rows: np.ndarray, kf: np.ndarray, scale: float, block_k: int) -> np.ndarray:
    """Eq. 5 for one query block given as its fp64 rows: vector over key blocks."""
    n = kf.shape[0]
    nbk = -(-n // block_k)
    s = scale * (q_rows @ kf.T)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)  # Eq. 1
    out = np.empty(nbk, dtype=np.float64)
    for c in range(nbk):
        out[c] = p[:, c * block_k : (c + 1) * block_k].sum() / p.shape[0]
    return out


def block_energy(q_bits: np.ndarray, k_bits: np.ndarray, scale: float, block_q: int, block_k: int) -> np.ndarray:
    """E[b, h, r, c] = mean over the queries of block r of the softmax mass they
    put on the keys of block c (Eq. 5).  fp64 [B, H, ceil(N/block_q), ceil(N/block_k)]."""
    B, H, N, D = q_bits.shape
    nbq, nbk = -(-N // block_q), -(-N // block_k)
    out = np.zeros((B, H, nbq, nbk), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            qf = bf16_bits_to_f64(q_bits[b, h])
            kf = bf16_bits_to_f64(k_bits[b, h])
            for r in range(nbq):
                out[b, h, r] = _energy_of_rows(qf[r * block_q : min((r + 1) * block_q, N)], kf, scale, block_k)
    return out


def block_energy_rows(q_bits, k_bits, scale: float, block_q: int, block_k: int, items):
    """Eq. 5 for selected block-rows only: for each (b, h, r) in ``items`` the
    fp64 vector over key blocks.  Same arithmetic as ``block_energy``."""
    N = q_bits.shape[2]
    out = []
    for (b, h, r) in items:
        qf = bf16_bits_to_f64(q_bits[b, h, r * block_q : min((r + 1) * block_q, N)])
        out.append(_energy_of_rows(qf, bf16_bits_to_f64(k_bits[b, h]), scale, block_k))
    return out


def select_row(energies, eps: float) -> np.ndarray:
    """Eq. 6 for one block-row: sort descending, keep the shortest prefix whose
    running sum reaches eps.  Returns a uint8 vector (1 = kept)."""
    e = [float(x) for x in energies]
    order = sorted(range(len(e)), key=lambda c: (-e[c], c))
    keep = np.zeros(len(e), dtype=np.uint8)
    total = 0.0
    for c in order:
        keep[c] = 1
        total += e[c]
        if total >= eps:
            break
    return keep


def select_blocks(E: np.ndarray, eps: float) -> np.ndarray:
    """Eq. 6 for every block-row of E[..., nbq, nbk]: uint8 mask of the same shape."""
    E = np.asarray(E)
    flat = E.reshape(-1, E.shape[-1])
    out = np.zeros(flat.shape, dtype=np.uint8)
    for i in range(flat.shape[0]):
        out[i] = select_row(flat[i], eps)
    return out.reshape(E.shape)


def epsilon_schedule(t: int, T: int, A: float, C: float, k: float) -> float:
    """Eq. 7: eps(t) = A + (C - A) exp(-k t / T), t = 0 the highest-noise step."""
    return A + (C - A) * math.exp(-k * t / T)


def schedule_base_level(N: int) -> float:
    """Base level A the paper uses in the many-step regime as a function of the
    sequence length (supplement Section A.1), together with C = 0.99, k = 16."""
    return 0.796 + 1.41e-6 * N


def schedule_constants(regime: int, N: int):
    """(A, C, k) of Eq. 7 as the supplement (Section A.1) gives them.  regime 0: the many-step models,
    A grows with the sequence length, C = 0.99, k = 16; regime 1: the few-step (distilled) models, one
    schedule for both resolutions, A = 0.763, C = 0.863, k = 5.64."""
    if regime == 0:
        return (0.796 + 1.41e-6 * N, 0.99, 16.0)
    if regime == 1:
        return (0.763, 0.863, 5.64)
    raise ValueError("regime 0 (many-step) or 1 (distilled)")


def flag_heads(scores, gamma: float):
    """Section 3.3: scores[p][h] = spatial similarity score of head h on calibration prompt p.  The
    scores are averaged over the prompts; a head is flagged as spatially repetitive when its average
    exceeds gamma.  Returns (flags uint8 [H], means float64 [H]); the mean adds the prompts in order."""
    rows = [[float(x) for x in row] for row in scores]
    n, H = len(rows), len(rows[0])
    means, flags = [], []
    for h in range(H):
        total = 0.0
        for p in range(n):
            total += rows[p][h]
        mean = total / n
        means.append(mean)
        flags.append(1 if mean > gamma else 0)
    return np.array(flags, dtype=np.uint8), np.array(means, dtype=np.float64)


def vote(masks: np.ndarray, rho: float) -> np.ndarray:
    """Eq. 8-9: masks[p, ...] of |D| prompts -> 1 where the fraction of prompts
    that kept the block is at least rho."""
    m = (np.asarray(masks) != 0).astype(np.float64)
    mean = m.sum(axis=0) / m.shape[0]
    return (mean >= rho).astype(np.uint8)
