"""Seeded, synthetic stand-ins for the paper's workloads.

The paper measures on video diffusion transformers (Wan 2.1 14B at 480p/720p,
Mochi 1; Section 4.1) with masks calibrated on real prompts.  None of those
models, prompts or masks are used here: only their *shapes* (Section B.1 of the
supplement: 21 latent frames of 30x52 tokens, 40 heads, head dim 128) and their
*mask statistics* (62-74 % sparsity in Tables 1-2; a few long runs of kept
blocks per row, supplement Fig. "Skip-list row length distribution"; large
intra-frame block structure, Fig. 2) are reproduced with a seeded generator.

Everything is drawn from ``numpy.random.default_rng(seed)`` (PCG64), in fp32 on
the host, and rounded to bf16 once; the resulting uint16 bit patterns are what
both the GPU path and the CPU oracle consume.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 20260305


# --------------------------------------------------------------------------
# bf16 bit helpers (input preparation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bits to fp32 exactly."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# token geometry
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Geometry:
    """Row-major video token grid: token = (frame * rows + y) * cols + x,
    followed by ``n_text`` text tokens (Mochi-style joint attention)."""

    frames: int
    rows: int
    cols: int
    n_text: int = 0

    @property
    def per_frame(self) -> int:
        return self.rows * self.cols

    @property
    def n_video(self) -> int:
        return self.frames * self.per_frame

    @property
    def n_tokens(self) -> int:
        return self.n_video + self.n_text


def _positional_code(geom: Geometry, n: int) -> np.ndarray:
    """Smooth rank-8 code of (frame, y, x): sin/cos at one frequency per axis
    plus one mixed term.  Text tokens get a constant code."""
    t = np.arange(n, dtype=np.int64)
    tv = np.minimum(t, max(geom.n_video - 1, 0))
    f = tv // geom.per_frame
    o = tv % geom.per_frame
    y = o // geom.cols
    x = o % geom.cols
    pf = 2.0 * np.pi * f / max(geom.frames, 1)
    py = 2.0 * np.pi * y / max(geom.rows, 1)
    px = 2.0 * np.pi * x / max(geom.cols, 1)
    code = np.stack(
        [np.sin(pf), np.cos(pf), np.sin(py), np.cos(py), np.sin(px), np.cos(px), np.sin(py + px), np.cos(py + px)],
        axis=1,
    ).astype(np.float32)
    if geom.n_text:
        code[t >= geom.n_video] = 0.0
    return code


def make_qkv(
    seed: int,
    B: int,
    H: int,
    N: int,
    D: int,
    geom: Optional[Geometry] = None,
    alpha: float = 0.0,
    qk_gain: float = 1.0,
) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q, k, v as uint16 bf16 bits, each [B, H, N, D].

    x = gain * (g + alpha * U[pos] W_h), g ~ N(0,1); q and k share the per-head
    projection W_h so that logits carry a positional component peaked at equal
    positions (attention concentrates on spatial neighbours and on the same
    patch across frames).  v ~ N(0,1).  ``alpha = 0`` gives plain N(0,1).
    """
    rng = np.random.default_rng(seed)
    out = [np.empty((B, H, N, D), dtype=np.uint16) for _ in range(3)]
    code = _positional_code(geom, N) if (geom is not None and alpha != 0.0) else None
    for b in range(B):
        for h in range(H):
            w = rng.standard_normal((8, D), dtype=np.float32) if code is not None else None
            for idx in range(3):
                g = rng.standard_normal((N, D), dtype=np.float32)
                if idx < 2:
                    if code is not None:
                        g += np.float32(alpha) * (code @ w)
                    if qk_gain != 1.0:
                        g *= np.float32(qk_gain)
                out[idx][b, h] = f32_to_bf16_bits(g)
    return out[0], out[1], out[2]


# --------------------------------------------------------------------------
# masks and repeat maps
# --------------------------------------------------------------------------
def tiny_mask(seed: int, H: int = 2, nb: int = 16, p_off: float = 0.3, n_repeat: int = 2):
    """Per head: |r-c| <= 1 band, block column 0, Bernoulli(p_off) elsewhere,
    diagonal always kept; ``n_repeat`` distinct query blocks in 1..nb-1 are
    marked as repeats of block 0."""
    rng = np.random.default_rng(seed)
    r = np.arange(nb)[:, None]
    c = np.arange(nb)[None, :]
    mask = np.zeros((H, nb, nb), dtype=np.uint8)
    repeat = np.full((H, nb), -1, dtype=np.int32)
    for h in range(H):
        m = (np.abs(r - c) <= 1) | (c == 0) | (rng.random((nb, nb)) < p_off)
        m[np.arange(nb), np.arange(nb)] = True
        mask[h] = m
        if n_repeat:
            rep = rng.choice(np.arange(1, nb), size=n_repeat, replace=False)
            repeat[h, rep] = 0
    return mask, repeat


def random_mask(seed: int, H: int, nbq: int, nbk: int, density: float, repeat_frac: float = 0.0,
                keep_diagonal: bool = False, allow_tail_source: bool = False, tail_partial: bool = False):
    """Unstructured Bernoulli mask and a random valid repeat map (test helper).

    A repeated block points at a non-repeated block of the same head; when
    ``tail_partial`` the last query block is shorter than the others, and unless
    ``allow_tail_source`` it is never used as a source."""
    rng = np.random.default_rng(seed)
    mask = (rng.random((H, nbq, nbk)) < density).astype(np.uint8)
    if keep_diagonal:
        for i in range(min(nbq, nbk)):
            mask[:, i, i] = 1
    repeat = np.full((H, nbq), -1, dtype=np.int32)
    n_rep = int(round(repeat_frac * nbq))
    n_rep = min(n_rep, nbq - 1)
    if n_rep > 0:
        for h in range(H):
            rep = rng.choice(nbq, size=n_rep, replace=False)
            is_rep = np.zeros(nbq, dtype=bool)
            is_rep[rep] = True
            src_ok = ~is_rep
            if tail_partial and not allow_tail_source:
                src_ok[nbq - 1] = False
            cand = np.flatnonzero(src_ok)
            if cand.size == 0:
                continue
            repeat[h, rep] = rng.choice(cand, size=n_rep, replace=True)
    return mask, repeat


def _smooth_noise(rng, n: int, corr: int) -> np.ndarray:
    z = rng.standard_normal(n + 2 * corr)
    ker = np.ones(2 * corr + 1) / (2 * corr + 1)
    s = np.convolve(z, ker, mode="valid")[:n]
    return s / (s.std() + 1e-9)


def calibrated_like_mask(
    seed: int,
    H: int,
    N: int,
    block: int,
    geom: Geometry,
    density: float,
    repeat_frac: float,
    repeat_mode: str = "uniform",
):
    """Band + temporal-stripe + sink mask with a global per-head top-k.

    Per head the block score is the larger of a spatial-band term (token
    distance inside one frame) and a temporal-stripe term (circular distance of
    the intra-frame offsets, slowly decaying with frame distance), divided by a
    smooth per-row temperature and jittered; sink columns and the diagonal are
    forced.  The best ``d_h * nb * nb`` blocks of the head are kept, so the
    per-row counts are uneven.  Head densities d_h vary around ``density``.
    Text blocks (any block touching a text token) are kept as whole rows and
    columns and the density target then refers to video-video blocks.

    Returns (mask uint8 [H,nb,nb], repeat int32 [H,nb], stats dict).
    """
    rng = np.random.default_rng(seed)
    nb = -(-N // block)
    per_frame = geom.per_frame
    n_video = geom.n_video
    centre = np.minimum(np.arange(nb, dtype=np.int64) * block + block // 2, N - 1)
    is_text = (np.arange(nb, dtype=np.int64) + 1) * block > n_video if geom.n_text else np.zeros(nb, dtype=bool)
    cv = np.minimum(centre, n_video - 1)
    frame = cv // per_frame
    off = cv % per_frame
    vid = np.flatnonzero(~is_text)
    nv = vid.size
    tail_partial = (N % block) != 0

    u = rng.uniform(0.5, 1.5, size=H)
    u = u / u.mean()
    d_h = np.clip(density * u, 0.02, 0.97)
    d_h = np.clip(d_h * (density / d_h.mean()), 0.02, 0.97)

    mask = np.zeros((H, nb, nb), dtype=np.uint8)
    repeat = np.full((H, nb), -1, dtype=np.int32)

    dtok = np.abs(cv[vid][:, None] - cv[vid][None, :]).astype(np.float64)
    same_frame = frame[vid][:, None] == frame[vid][None, :]
    doff = np.abs(off[vid][:, None] - off[vid][None, :]).astype(np.float64)
    doff = np.minimum(doff, per_frame - doff)
    dfr = np.abs(frame[vid][:, None] - frame[vid][None, :]).astype(np.float64)

    if repeat_mode == "paperlike" and repeat_frac > 0:
        # repetition concentrated in few heads, ~5/6 of their blocks repeated
        n_heads_rep = max(1, int(round(repeat_frac * H / (5.0 / 6.0))))
        rep_heads = set(rng.choice(H, size=min(n_heads_rep, H), replace=False).tolist())
    else:
        rep_heads = None

    for h in range(H):
        w_band = block * math.exp(rng.uniform(math.log(1.0), math.log(6.0)))
        w_stripe = block * math.exp(rng.uniform(math.log(0.4), math.log(2.5)))
        beta = rng.uniform(0.02, 0.4)
        n_sink = int(rng.integers(1, 3))
        temp = np.exp(0.45 * _smooth_noise(rng, nv, max(2, nv // 24)))
        band = np.where(same_frame, -dtok / w_band, -np.inf)
        stripe = -(doff / w_stripe + beta * dfr)
        score = np.maximum(band, stripe) / temp[:, None]
        score += 0.15 * rng.standard_normal((nv, nv))
        forced = np.zeros((nv, nv), dtype=bool)
        forced[np.arange(nv), np.arange(nv)] = True
        forced[:, :n_sink] = True
        dense_head = rep_heads is not None and h in rep_heads
        k_keep = nv * nv if dense_head else int(round(d_h[h] * nv * nv))
        k_keep = max(k_keep, int(forced.sum()))
        score[forced] = np.inf
        flat = score.ravel()
        keep = np.zeros(nv * nv, dtype=bool)
        if k_keep >= nv * nv:
            keep[:] = True
        else:
            keep[np.argpartition(-flat, k_keep - 1)[:k_keep]] = True
        m = np.zeros((nb, nb), dtype=np.uint8)
        m[np.ix_(vid, vid)] = keep.reshape(nv, nv)
        if geom.n_text:
            m[is_text, :] = 1
            m[:, is_text] = 1
        mask[h] = m

        # repeat map
        eligible = ~is_text
        if tail_partial:
            eligible = eligible.copy()
            eligible[nb - 1] = False
        elig = np.flatnonzero(eligible)
        if rep_heads is None:
            n_rep = int(round(repeat_frac * nb))
        else:
            n_rep = int(round((5.0 / 6.0) * elig.size)) if dense_head else 0
        n_rep = min(n_rep, elig.size - 1)
        if n_rep > 0:
            rep = rng.choice(elig, size=n_rep, replace=False)
            is_rep = np.zeros(nb, dtype=bool)
            is_rep[rep] = True
            src_cand = np.flatnonzero(eligible & ~is_rep)
            for r in rep:
                same = src_cand[frame[src_cand] == frame[r]]
                pool = same if same.size else src_cand
                repeat[h, r] = int(pool[np.argmin(np.abs(pool - r))])

    kept_rows = mask.sum(axis=2)
    stats = {
        "density": float(mask.mean()),
        "density_video": float(mask[:, vid][:, :, vid].mean()),
        "row_min": int(kept_rows.min()),
        "row_median": float(np.median(kept_rows)),
        "row_max": int(kept_rows.max()),
        "repeat_frac": float((repeat >= 0).mean()),
    }
    return mask, repeat, stats


def runs_per_row(mask: np.ndarray) -> np.ndarray:
    """Number of maximal runs of kept blocks in every mask row (a statistic the
    paper plots for its calibrated masks; used to sanity-check the generator)."""
    m = (mask != 0).astype(np.int8)
    starts = m[..., :1].astype(np.int64).sum(axis=-1) + ((m[..., 1:] - m[..., :-1]) == 1).sum(axis=-1)
    return starts


# --------------------------------------------------------------------------
# named configurations
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    B: int
    H: int
    N: int
    D: int
    block_q: int
    block_k: int
    scale: float
    mask: np.ndarray
    repeat: np.ndarray
    q: Optional[np.ndarray] = None
    k: Optional[np.ndarray] = None
    v: Optional[np.ndarray] = None
    stats: Dict = field(default_factory=dict)
    geometry: Optional[tuple] = None  # (frames, rows per frame, columns) of the video tokens

    @property
    def nbq(self) -> int:
        return -(-self.N // self.block_q)

    @property
    def nbk(self) -> int:
        return -(-self.N // self.block_k)


CONFIGS = {
    # name: (index, B, H, D, block, geometry, density, repeat fraction, alpha)
    "tiny": dict(index=0, B=1, H=2, D=64, block=64, geom=Geometry(1, 32, 32), density=None, repeat=None, alpha=0.0),
    "wan480": dict(index=1, B=1, H=40, D=128, block=128, geom=Geometry(21, 30, 52), density=0.30, repeat=0.10, alpha=0.4),
    "wan720": dict(index=2, B=1, H=40, D=128, block=128, geom=Geometry(21, 45, 80), density=0.30, repeat=0.20, alpha=0.4),
    "mochi": dict(index=3, B=1, H=24, D=128, block=128, geom=Geometry(28, 30, 53, n_text=256), density=0.25, repeat=0.15, alpha=0.4),
}


def make_workload(
    name: str,
    variant: int = 0,
    density: Optional[float] = None,
    repeat_frac: Optional[float] = None,
    with_qkv: bool = True,
    heads: Optional[int] = None,
    qk_gain: float = 1.0,
    repeat_mode: str = "uniform",
    dense: bool = False,
) -> Workload:
    """Build one of the named configurations.  ``dense=True`` replaces the mask
    by all-ones without repeats (the dense reference run); ``heads`` overrides
    the head count (smaller parity cases of the same shape)."""
    cfg = CONFIGS[name]
    seed = BASE_SEED + 1000 * cfg["index"] + variant
    geom: Geometry = cfg["geom"]
    H = heads if heads is not None else cfg["H"]
    N, D, blk = geom.n_tokens, cfg["D"], cfg["block"]
    stats: Dict = {}
    nb = -(-N // blk)
    if dense:
        mask = np.ones((H, nb, nb), dtype=np.uint8)
        repeat = np.full((H, nb), -1, dtype=np.int32)
        stats = {"density": 1.0, "repeat_frac": 0.0}
    elif name == "tiny":
        mask, repeat = tiny_mask(seed, H=H, nb=nb)
        stats = {"density": float(mask.mean()), "repeat_frac": float((repeat >= 0).mean())}
    else:
        d = cfg["density"] if density is None else density
        p = cfg["repeat"] if repeat_frac is None else repeat_frac
        mask, repeat, stats = calibrated_like_mask(seed, H, N, blk, geom, d, p, repeat_mode=repeat_mode)
    wl = Workload(name, cfg["B"], H, N, D, blk, blk, 1.0 / math.sqrt(D), mask, repeat, stats=stats,
                  geometry=(geom.frames, geom.rows, geom.cols))
    if with_qkv:
        wl.q, wl.k, wl.v = make_qkv(seed + 500, cfg["B"], H, N, D, geom, alpha=cfg["alpha"], qk_gain=qk_gain)
    return wl


def sweep_pattern(layer: int, step: int, heads: int = 40):
    """Pattern of one (layer, timestep) of the full-step sweep at the Wan-480p
    shape: density ~ U(0.1, 0.6), repeat fraction ~ U(0, 0.3), distinct seed."""
    cfg = CONFIGS["wan480"]
    seed = BASE_SEED + 1000 * 4 + 50 * layer + step
    rng = np.random.default_rng(seed)
    d = float(rng.uniform(0.1, 0.6))
    p = float(rng.uniform(0.0, 0.3))
    geom: Geometry = cfg["geom"]
    mask, repeat, stats = calibrated_like_mask(seed + 100000, heads, geom.n_tokens, cfg["block"], geom, d, p)
    return mask, repeat, stats


def dictionary_head_masks(layer: int, head: int, steps: int = 50, name: str = "wan720") -> np.ndarray:
    """Masks of one (layer, head) over the timesteps of a generation, uint8 [steps, nb, nb]: a
    synthetic stand-in for a calibrated dictionary whose masks resemble each other more and more
    at later timesteps (supplement A.3).  One block score per head (spatial band and temporal
    stripe as in ``calibrated_like_mask``), a kept fraction that falls with the timestep as the
    many-step energy schedule does (exp(-16 t/T), supplement A.1), and a small score jitter per
    step so that neighbouring steps differ in a few blocks.  Diagonal and one sink column forced."""
    cfg = CONFIGS[name]
    geom: Geometry = cfg["geom"]
    N, block = geom.n_tokens, cfg["block"]
    nb = -(-N // block)
    rng = np.random.default_rng(BASE_SEED + 700000 + 1000 * layer + head)
    centre = np.minimum(np.arange(nb, dtype=np.int64) * block + block // 2, geom.n_video - 1)
    frame, off = centre // geom.per_frame, centre % geom.per_frame
    dtok = np.abs(centre[:, None] - centre[None, :]).astype(np.float64)
    doff = np.abs(off[:, None] - off[None, :]).astype(np.float64)
    doff = np.minimum(doff, geom.per_frame - doff)
    dfr = np.abs(frame[:, None] - frame[None, :]).astype(np.float64)
    w_band = block * math.exp(rng.uniform(math.log(1.0), math.log(6.0)))
    w_stripe = block * math.exp(rng.uniform(math.log(0.4), math.log(2.5)))
    beta = rng.uniform(0.02, 0.4)
    temp = np.exp(0.45 * _smooth_noise(rng, nb, max(2, nb // 24)))
    band = np.where(frame[:, None] == frame[None, :], -dtok / w_band, -np.inf)
    base = np.maximum(band, -(doff / w_stripe + beta * dfr)) / temp[:, None] + 0.15 * rng.standard_normal((nb, nb))
    base[np.arange(nb), np.arange(nb)] = np.inf
    base[:, 0] = np.inf
    d_late = float(np.clip(cfg["density"] * rng.uniform(0.5, 1.5), 0.05, 0.9))
    out = np.zeros((steps, nb, nb), dtype=np.uint8)
    for t in range(steps):
        d_t = d_late + (0.95 - d_late) * math.exp(-16.0 * t / steps)
        score = base + 0.02 * rng.standard_normal((nb, nb))
        k_keep = max(int(round(d_t * nb * nb)), 2 * nb)
        flat = score.ravel()
        keep = np.zeros(nb * nb, dtype=bool)
        keep[np.argpartition(-flat, k_keep - 1)[:k_keep]] = True
        out[t] = keep.reshape(nb, nb)
    return out
