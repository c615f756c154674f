"""fp64 definition of the spatial-row anchor scheme (paper, Section 3.3 and the
"Inference stage" paragraph of Section 3.4).

TEST INFRASTRUCTURE ONLY - never imported by the product package.

Setting: the first F*Hs*Ws tokens of a head are a video latent, token
(f, y, x) at index (f*Hs + y)*Ws + x, i.e. frame, then spatial row, then
column.  Tokens after them (text tokens of a joint-attention model) have no
spatial position.

What is computed for a head flagged as spatially repetitive:

* k anchor spatial rows are chosen per frame, equally spaced.  The paper does
  not print the positions; the reading taken here: cut the Hs rows into k
  equal real-valued segments and take the row under each segment's centre,
  a_j = floor((2j + 1) * Hs / (2k)), j = 0..k-1.
* the queries of the anchor rows attend to ALL N keys and values with the
  plain softmax of Section 2, Eq. 1-2 (the paper runs its dense kernel on the
  reduced query set);
* every spatial row y of a frame takes the output of its nearest anchor row of
  the same frame, column by column: out[f, y, x] = A[f, a(y), x] with
  a(y) = argmin_j |y - a_j|, the lower row winning a tie (the paper leaves ties
  open);
* tokens without a spatial position are computed from their own query.

Nothing is tiled or reordered: the anchor queries' logits against all keys are
materialised and pushed through a max-subtracted softmax.

Detection (Section 3.3, second paragraph): the spatial similarity score of a
head is the cosine similarity between the flattened attention rows of a spatial
row, P^(f,i) = flatten(P[I^(f,i), :]) (Ws tokens x N keys), and those of its
nearest anchor row, averaged over frames f and spatial rows i.  Reading: the
average runs over every spatial row, anchors included (their similarity is 1);
a head is flagged when the score, further averaged over prompts by the caller,
exceeds the threshold gamma.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

from .attention import bf16_bits_to_f64


def anchor_rows(n_rows: int, k: int) -> np.ndarray:
    """Row indices of the k equally spaced anchors among ``n_rows`` rows."""
    if not (1 <= k <= n_rows):
        raise ValueError("need 1 <= k <= rows per frame")
    return np.array([((2 * j + 1) * n_rows) // (2 * k) for j in range(k)], dtype=np.int64)


def nearest_anchor(n_rows: int, k: int) -> np.ndarray:
    """For every spatial row y the index j of its nearest anchor row (ties: the
    lower anchor)."""
    a = anchor_rows(n_rows, k)
    out = np.empty(n_rows, dtype=np.int64)
    for y in range(n_rows):
        best = 0
        for j in range(1, k):
            if abs(y - int(a[j])) < abs(y - int(a[best])):
                best = j
        out[y] = best
    return out


def anchor_token_maps(N: int, F: int, Hs: int, Ws: int, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """(q_index, src): q_index[i] is the token whose query is the i-th computed
    one (frames ascending, then anchors ascending, then columns; after them the
    tokens without a spatial position, ascending); src[t] is the position in
    q_index of the computed query whose output token t receives."""
    n_video = F * Hs * Ws
    if min(N, F, Hs, Ws) <= 0 or n_video > N:
        raise ValueError("video tokens F*Hs*Ws must fit in N")
    a = anchor_rows(Hs, k)
    near = nearest_anchor(Hs, k)
    q_index = []
    for f in range(F):
        for j in range(k):
            for x in range(Ws):
                q_index.append((f * Hs + int(a[j])) * Ws + x)
    for t in range(n_video, N):
        q_index.append(t)
    src = np.empty(N, dtype=np.int64)
    for f in range(F):
        for y in range(Hs):
            for x in range(Ws):
                src[(f * Hs + y) * Ws + x] = (f * k + int(near[y])) * Ws + x
    for t in range(n_video, N):
        src[t] = F * k * Ws + (t - n_video)
    return np.array(q_index, dtype=np.int64), src


def dense_rows(qf: np.ndarray, kf: np.ndarray, vf: np.ndarray, scale: float) -> np.ndarray:
    """softmax(scale * q K^T) V for the given query rows against all keys
    (Section 2, Eq. 1-2)."""
    s = scale * (qf @ kf.T)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return (e / e.sum(axis=1, keepdims=True)) @ vf


def anchor_attention(
    q_bits: np.ndarray,
    k_bits: np.ndarray,
    v_bits: np.ndarray,
    heads: Sequence[int],
    F: int,
    Hs: int,
    Ws: int,
    k: int,
    scale: float,
    chunk: int = 2048,
) -> np.ndarray:
    """Output of the listed heads, fp64 [B, len(heads), N, D].  q/k/v: uint16
    bf16 bits [B, H, N, D].  ``chunk`` only bounds the size of the logits held
    at once; every row is an independent softmax, so it changes no value."""
    B, H, N, D = q_bits.shape
    q_index, src = anchor_token_maps(N, F, Hs, Ws, k)
    out = np.zeros((B, len(heads), N, D), dtype=np.float64)
    for b in range(B):
        for i, h in enumerate(heads):
            qf = bf16_bits_to_f64(q_bits[b, h])[q_index]
            kf = bf16_bits_to_f64(k_bits[b, h])
            vf = bf16_bits_to_f64(v_bits[b, h])
            a = np.empty((q_index.size, D), dtype=np.float64)
            for lo in range(0, q_index.size, chunk):
                a[lo : lo + chunk] = dense_rows(qf[lo : lo + chunk], kf, vf, scale)
            out[b, i] = a[src]
    return out


def spatial_similarity(q_bits: np.ndarray, k_bits: np.ndarray, F: int, Hs: int, Ws: int, k: int, scale: float) -> np.ndarray:
    """Score s[b, h] of every head (Section 3.3): mean over frames and spatial
    rows of cos(P^(f,i), P^(f,a(i))).  Materialises P of the video tokens: small
    inputs only."""
    B, H, N, D = q_bits.shape
    n_video = F * Hs * Ws
    a = anchor_rows(Hs, k)
    near = nearest_anchor(Hs, k)
    out = np.zeros((B, H), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            qf = bf16_bits_to_f64(q_bits[b, h, :n_video])
            kf = bf16_bits_to_f64(k_bits[b, h])
            s = scale * (qf @ kf.T)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)           # Eq. 1, [n_video, N]
            p = p.reshape(F, Hs, Ws * N)                    # P^(f,i) flattened
            total = 0.0
            for f in range(F):
                for i in range(Hs):
                    u, w = p[f, i], p[f, int(a[near[i]])]
                    total += float(u @ w) / (np.sqrt(float(u @ u)) * np.sqrt(float(w @ w)))
            out[b, h] = total / (F * Hs)
    return out


def spatial_similarity_rows(q_bits, k_bits, F: int, Hs: int, Ws: int, k: int, scale: float, items) -> list:
    """cos(P^(f,i), P^(f,a(i))) of selected spatial rows only: ``items`` holds
    (b, h, f, i).  Same arithmetic as ``spatial_similarity``, whose score is the
    mean of these values over all (f, i)."""
    a = anchor_rows(Hs, k)
    near = nearest_anchor(Hs, k)
    out = []
    for (b, h, f, i) in items:
        kf = bf16_bits_to_f64(k_bits[b, h])

        def flat_probs(row):
            t0 = (f * Hs + row) * Ws
            s = scale * (bf16_bits_to_f64(q_bits[b, h, t0 : t0 + Ws]) @ kf.T)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            return (p / p.sum(axis=1, keepdims=True)).reshape(-1)

        u, w = flat_probs(i), flat_probs(int(a[near[i]]))
        out.append(float(u @ w) / (np.sqrt(float(u @ u)) * np.sqrt(float(w @ w))))
    return out
