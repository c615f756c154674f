"""Calibration and inference stages wired together (paper, Section 3.4) on top of
the C ABI.  Orchestration only: every computation and every decision is a library call.

``Calibrator`` collects, per (timestep, layer) key and over calibration prompts,
the votes of the per-prompt block masks (Section 3.2: block energy, selection at
eps(t); one uint16 counter per block, no mask is kept) and
the spatial similarity scores of the heads (Section 3.3); ``finalize`` votes the
masks (Eq. 8-9) and flags the heads whose mean score exceeds gamma.

``CalibAttention`` is the dictionary that stays on the GPU at inference: per key
a compiled pattern over the heads that are not flagged (interval form by
default) and the list of flagged heads, which go through the anchor-row path.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Hashable, List, Optional, Sequence, Tuple

import numpy as np

from . import binding as _b


@dataclass
class CalibrationResult:
    mask: np.ndarray              # uint8 [H, nbq, nbk], 1 = kept
    repetitive_heads: List[int]   # heads that take the anchor-row path
    scores: Optional[np.ndarray]  # mean spatial similarity per head, or None
    n_prompts: int


class Calibrator:
    def __init__(self, H: int, N: int, D: int, block_q: int = 128, block_k: int = 128,
                 geometry: Optional[Tuple[int, int, int]] = None, anchors: int = 5,
                 rho: float = 0.5, gamma: float = 0.87):
        self.H, self.N, self.D = H, N, D
        self.block_q, self.block_k = block_q, block_k
        self.geometry, self.anchors, self.rho, self.gamma = geometry, anchors, rho, gamma
        self._counts: Dict[Hashable, object] = {}       # CUDA tensor, uint16 per block: prompts that kept it
        self._n: Dict[Hashable, int] = {}
        self._scores: Dict[Hashable, List[np.ndarray]] = {}
        self._partner = None
        self._energy_workspace = None   # of the one-pass energy kernel; calls are issued on one stream

    def observe(self, key: Hashable, q, k, eps: float, scale: float) -> None:
        """One dense forward's q, k ([B, H, N, D] bf16 CUDA tensors; every batch element counts as a
        prompt) at the step/layer ``key``, with the energy threshold ``eps`` of that step."""
        import torch

        # energy -> Eq. 6 -> one more vote per block, all on the device; the counters come back in finalize
        if self._energy_workspace is None or self._energy_workspace.device != q.device:
            nbytes = _b.block_energy_workspace_bytes(self.N, self.block_q, self.block_k)
            self._energy_workspace = torch.empty(nbytes // 4, dtype=torch.float32, device=q.device)
        energy = _b.block_energy(q, k, self.block_q, self.block_k, scale, workspace=self._energy_workspace)
        masks = _b.select_blocks_device(energy, eps)  # [B, H, nbq, nbk]
        if self._n.get(key, 0) + masks.shape[0] > 65535:
            raise ValueError("at most 65535 prompts per key")
        if key not in self._counts:
            self._counts[key] = torch.zeros(masks.shape[1:], dtype=torch.int16, device=q.device)  # uint16 counters
        for b in range(masks.shape[0]):
            _b.vote_accumulate_device(masks[b], self._counts[key])
        self._n[key] = self._n.get(key, 0) + masks.shape[0]
        if self.geometry is not None:
            F, Hs, Ws = self.geometry
            if self._partner is None:
                self._partner = torch.from_numpy(_b.anchor_partner(F, Hs, Ws, self.anchors)).to(q.device)
            score = _b.spatial_similarity(q, k, self._partner, Ws, scale).cpu().numpy()
            self._scores.setdefault(key, []).extend(score[b] for b in range(score.shape[0]))

    def finalize(self, merge_percentile: Optional[float] = None) -> Dict[Hashable, CalibrationResult]:
        out = {}
        for key, counts in self._counts.items():
            mask = _b.vote_finish(counts.cpu().numpy().view(np.uint16), self._n[key], self.rho)
            if merge_percentile is not None:
                mask, _ = _b.merge_intervals(mask, merge_percentile)
            scores, flagged = None, []
            if key in self._scores:
                flags, scores = _b.flag_heads(np.stack(self._scores[key]), self.gamma)  # mean over prompts vs gamma
                flagged = [h for h in range(self.H) if flags[h]]
            out[key] = CalibrationResult(mask=mask, repetitive_heads=flagged, scores=scores, n_prompts=self._n[key])
        return out


def save_calibration(path: str, results: Dict[Hashable, CalibrationResult]) -> None:
    """Writes the calibrated masks and flags to one .npz file (block masks bit-packed).  Keys must be
    tuples of integers, e.g. (timestep, layer)."""
    arrays = {}
    keys = sorted(results)
    arrays["keys"] = np.array([list(k) for k in keys], dtype=np.int64).reshape(len(keys), -1)
    for i, key in enumerate(keys):
        res = results[key]
        arrays[f"mask_shape_{i}"] = np.array(res.mask.shape, dtype=np.int64)
        arrays[f"mask_bits_{i}"] = np.packbits(np.asarray(res.mask, dtype=np.uint8).reshape(-1) != 0)
        arrays[f"heads_{i}"] = np.array(res.repetitive_heads, dtype=np.int32)
        arrays[f"scores_{i}"] = np.zeros(0) if res.scores is None else np.asarray(res.scores, dtype=np.float64)
        arrays[f"prompts_{i}"] = np.array([res.n_prompts], dtype=np.int64)
    np.savez_compressed(path, **arrays)


def load_calibration(path: str) -> Dict[Hashable, CalibrationResult]:
    """Inverse of ``save_calibration`` (plain arrays only, nothing is unpickled)."""
    out = {}
    with np.load(path, allow_pickle=False) as z:
        for i, key in enumerate(z["keys"]):
            shape = tuple(int(x) for x in z[f"mask_shape_{i}"])
            n = int(np.prod(shape))
            mask = np.unpackbits(z[f"mask_bits_{i}"])[:n].reshape(shape).astype(np.uint8)
            scores = z[f"scores_{i}"]
            out[tuple(int(x) for x in key)] = CalibrationResult(
                mask=mask, repetitive_heads=[int(h) for h in z[f"heads_{i}"]],
                scores=None if scores.size == 0 else scores, n_prompts=int(z[f"prompts_{i}"][0]))
    return out


@dataclass
class _Entry:
    pattern: Optional[_b.DevicePattern]
    head_ids: Optional[object]  # int32 CUDA tensor of the flagged heads, or None
    kept_blocks: int = 0
    sparse_heads: List[int] = field(default_factory=list)


class CalibAttention:
    def __init__(self, H: int, N: int, D: int, block_q: int = 128, block_k: int = 128,
                 geometry: Optional[Tuple[int, int, int]] = None, anchors: int = 5,
                 intervals: bool = True, order: int = 4, device: str = "cuda"):
        self.H, self.N, self.D = H, N, D
        self.block_q, self.block_k = block_q, block_k
        self.intervals, self.order, self.device = intervals, order, device
        self.entries: Dict[Hashable, _Entry] = {}
        self.amap = None
        self._anchor_workspace: Dict[Tuple[int, int, int], object] = {}
        if geometry is not None:
            F, Hs, Ws = geometry
            self.amap = _b.anchor_map(N, F, Hs, Ws, anchors).to_device(device)

    def add(self, key: Hashable, mask, repetitive_heads: Sequence[int] = (), repeat=None) -> None:
        """Compile and upload the pattern of ``key``.  ``mask`` [H, nbq, nbk]; ``repetitive_heads`` take
        the anchor-row path (needs a geometry); ``repeat`` is the optional block-level repeat map."""
        import torch

        flagged = sorted(set(int(h) for h in repetitive_heads))
        if flagged and self.amap is None:
            raise ValueError("repetitive heads need the token geometry")
        sparse = [h for h in range(self.H) if h not in flagged]
        m = np.asarray(mask)
        pattern, kept = None, 0
        if sparse:
            rep = None if repeat is None else np.asarray(repeat)[sparse]
            hp = _b.compile_pattern(m[sparse], rep, len(sparse), self.N, self.block_q, self.block_k, self.order)
            head_map = None if len(sparse) == self.H else sparse
            pattern = hp.to_device(self.device, intervals=self.intervals, head_map=head_map)
            kept = hp.nnz
        head_ids = torch.tensor(flagged, dtype=torch.int32, device=self.device) if flagged else None
        self.entries[key] = _Entry(pattern, head_ids, kept, sparse)

    def add_calibrated(self, results: Dict[Hashable, CalibrationResult], share_tau: Optional[float] = None) -> None:
        """Adds every calibrated key.  ``share_tau``: timestep mask sharing (supplement A.3).  Keys must
        then be (timestep, layer) pairs; per layer and head the timesteps are clustered by
        ``calibatt_share_timesteps`` (IoU of the skipped-block sets >= tau with every member of the
        cluster) and every member takes the cluster's shared mask.  Keys of a layer whose masks and flagged
        heads then coincide are stored once: they share one compiled pattern on the GPU."""
        masks = {key: np.asarray(res.mask, dtype=np.uint8) for key, res in results.items()}
        if share_tau is not None:
            layers = sorted({key[1] for key in results})
            for layer in layers:
                steps = sorted(key[0] for key in results if key[1] == layer)
                stack = np.stack([masks[(t, layer)] for t in steps])  # [T, H, nbq, nbk]
                shared = np.empty_like(stack)
                for h in range(stack.shape[1]):
                    cluster, cluster_masks = _b.share_timesteps(stack[:, h], share_tau)
                    shared[:, h] = cluster_masks[cluster]
                for i, t in enumerate(steps):
                    masks[(t, layer)] = shared[i]
        stored: Dict[Tuple, Hashable] = {}
        for key, res in results.items():
            layer = key[1] if share_tau is not None else key
            fingerprint = (layer, tuple(res.repetitive_heads), masks[key].shape, np.packbits(masks[key]).tobytes())
            if share_tau is not None and fingerprint in stored:
                self.entries[key] = self.entries[stored[fingerprint]]  # one device pattern for the cluster
                continue
            self.add(key, masks[key], res.repetitive_heads)
            stored[fingerprint] = key

    def __call__(self, q, k, v, out, key: Hashable, scale: float, stream=None):
        """One attention call of step/layer ``key``: the sparse forward on the heads of the pattern,
        the anchor-row forward on the flagged heads; together they write every head of ``out``."""
        e = self.entries[key]
        if e.pattern is not None:
            _b.sparse_attn_fwd(q, k, v, out, e.pattern, scale, stream=stream)
        if e.head_ids is not None:
            _b.anchor_attn_fwd(q, k, v, out, e.head_ids, self.amap, scale, stream=stream,
                               workspace=self._workspace_for(q, e.head_ids.numel(), stream))
        return out

    def _workspace_for(self, q, n_heads: int, stream):
        """Workspace of the key-range split of the anchor path, one per (batch, flagged heads, stream):
        calls on one stream run in order and may share it, calls on different streams may overlap."""
        import torch

        handle = torch.cuda.current_stream(q.device).cuda_stream if stream is None else int(stream)
        key = (q.shape[0], n_heads, handle)
        if key not in self._anchor_workspace:
            with torch.cuda.device(q.device):
                n_split, nbytes = _b.anchor_split_plan(q.shape[0], self.N, self.D, n_heads, self.amap.n_q)
            self._anchor_workspace[key] = (torch.empty(nbytes // 4, dtype=torch.float32, device=q.device)
                                           if n_split > 1 else None)
        return self._anchor_workspace[key]

    @property
    def index_bytes(self) -> int:
        """Bytes of kept-block lists resident on the GPU (a pattern shared by several keys counts once)."""
        unique = {id(e): e for e in self.entries.values()}
        return sum(e.pattern.index_bytes for e in unique.values() if e.pattern is not None)

    @property
    def index_bytes_unshared(self) -> int:
        """The same with every key holding a pattern of its own."""
        return sum(e.pattern.index_bytes for e in self.entries.values() if e.pattern is not None)
