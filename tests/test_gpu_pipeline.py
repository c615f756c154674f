"""End to end on the GPU: calibrate on synthetic prompts (block energy ->
selection -> vote; spatial similarity -> flags), build the resident dictionary,
run inference attention through both paths, compare with dense attention.

The synthetic "model": heads 0-1 have queries that do not depend on the spatial
row (the structure Section 3.3 exploits), heads 2-3 have queries and keys with a
strong positional component, so that their attention mass sits in few blocks
(the structure Section 3.2 exploits).  Each prompt is a new seed of the same
structure."""
import math

import numpy as np
import pytest

from oracle import anchor_attention, sparse_attention
from tests.parity_utils import MAX_ABS, bits_to_f64, from_dev, to_dev
from workloads import f32_to_bf16_bits

pytestmark = pytest.mark.gpu

F, HS, WS, D, H, BLK = 3, 8, 32, 64, 4, 64
N = F * HS * WS


def _prompt(seed):
    rng = np.random.default_rng(seed)
    pos = np.arange(N)
    code = np.stack([np.sin(2 * np.pi * pos / N * f) for f in (1, 2, 3, 5)] +
                    [np.cos(2 * np.pi * pos / N * f) for f in (1, 2, 3, 5)], axis=1)  # [N, 8]
    proj = np.random.default_rng(1234).standard_normal((8, D))  # the "weights": shared by all prompts
    q = rng.standard_normal((H, N, D))
    k = rng.standard_normal((H, N, D))
    for h in (2, 3):
        q[h] = 0.3 * q[h] + 4.0 * code @ proj
        k[h] = 0.3 * k[h] + 4.0 * code @ proj
    for h in (0, 1):
        base = 1.5 * rng.standard_normal((F, 1, WS, D))
        q[h] = np.broadcast_to(base, (F, HS, WS, D)).reshape(N, D)
    v = rng.standard_normal((H, N, D))
    return tuple(f32_to_bf16_bits(x[None].astype(np.float32)) for x in (q, k, v))


def test_calibrate_then_infer(lib):
    import torch

    print("pipeline", flush=True)
    scale = 1 / math.sqrt(D)
    cal = lib.Calibrator(H, N, D, BLK, BLK, geometry=(F, HS, WS), anchors=2, rho=0.5, gamma=0.87)
    T = 4
    A = lib.schedule_base_level(N)
    for prompt in range(4):
        q, k, _ = _prompt(100 + prompt)
        for t in (0, 3):
            cal.observe(("t", t), to_dev(q), to_dev(k), lib.epsilon_schedule(t, T, A, 0.99, 16.0), scale)
    results = cal.finalize()
    assert set(results) == {("t", 0), ("t", 3)}
    for key, res in results.items():
        print(key, "scores", np.round(res.scores, 3), "flagged", res.repetitive_heads,
              "density per head", np.round(res.mask.mean(axis=(1, 2)), 3), flush=True)
        assert res.n_prompts == 4 and res.repetitive_heads == [0, 1]
        assert res.mask[2:].mean() < 0.6  # the positional heads concentrate their mass
    # a later step has a lower threshold: never denser
    assert results[("t", 3)].mask[2:].sum() <= results[("t", 0)].mask[2:].sum()

    att = lib.CalibAttention(H, N, D, BLK, BLK, geometry=(F, HS, WS), anchors=2)
    att.add_calibrated(results)
    q, k, v = _prompt(999)  # an unseen prompt
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    dense = sparse_attention(q, k, v, np.ones((H, N // BLK, N // BLK), np.uint8), None, scale, BLK, BLK)
    for key, res in results.items():
        out = torch.empty_like(tq)
        out.view(torch.int16).fill_(0x7FC1)
        att(tq, tk, tv, out, key, scale)
        torch.cuda.synchronize()
        got = bits_to_f64(from_dev(out))
        assert np.isfinite(got).all()
        # parity against the oracle of what was asked for: anchor path on heads 0-1, masked attention on 2-3
        want_anchor = anchor_attention(q, k, v, [0, 1], F, HS, WS, 2, scale)
        assert np.abs(got[:, :2] - want_anchor).max() <= MAX_ABS
        want_sparse = sparse_attention(q[:, 2:], k[:, 2:], v[:, 2:], res.mask[2:], None, scale, BLK, BLK)
        assert np.abs(got[:, 2:] - want_sparse).max() <= MAX_ABS
        # and the approximation itself stays close to dense attention
        rel = [np.linalg.norm(got[0, h] - dense[0, h]) / np.linalg.norm(dense[0, h]) for h in range(H)]
        print(key, "relative L2 distance to dense attention per head", np.round(rel, 4), flush=True)
        assert max(rel[:2]) < 0.02  # rows repeat exactly: only rounding
        # up to 1 - eps of every row's mass is dropped: eps = 0.99 at step 0, 0.84 at the last step
        assert max(rel[2:]) < (0.08 if key == ("t", 0) else 0.6)


def test_timestep_sharing_and_two_streams_on_one_key(lib):
    """Timestep mask sharing in the resident dictionary (supplement A.3): timesteps whose skipped sets
    overlap enough take the cluster's OR mask and share one device pattern.  And the same key called on
    two streams at once (the two guidance branches) gives each call's bits: the wrapper hands every
    stream scheduler counters of its own."""
    import torch

    from workloads import random_mask

    print("pipeline sharing", flush=True)
    Hh, Nn, Dd, blk = 3, 64 * 40 + 17, 64, 64
    nb = -(-Nn // blk)
    rng = np.random.default_rng(5)
    base, _ = random_mask(11, Hh, nb, nb, 0.5, 0.0)
    results = {}
    for t in range(6):
        m = base.copy()
        if t >= 3:                       # the late steps drop a quarter of the blocks: a second cluster
            drop = np.random.default_rng(77).random(m.shape) < 0.5
            m[drop] = 0
        flip = rng.random(m.shape) < 0.002 * (t % 3)   # small differences inside a cluster
        m[flip] = 0
        m[:, np.arange(nb), np.arange(nb)] = 1
        results[(t, 0)] = lib.CalibrationResult(mask=m, repetitive_heads=[], scores=None, n_prompts=1)
    att = lib.CalibAttention(Hh, Nn, Dd, blk, blk)
    att.add_calibrated(results, share_tau=0.9)
    patterns = {id(att.entries[(t, 0)]) for t in range(6)}
    assert len(patterns) == 2 and att.entries[(0, 0)] is att.entries[(2, 0)] and att.entries[(3, 0)] is att.entries[(5, 0)]
    assert att.index_bytes * 3 == att.index_bytes_unshared
    shared_mask = results[(0, 0)].mask | results[(1, 0)].mask | results[(2, 0)].mask
    q = f32_to_bf16_bits((2.0 * rng.standard_normal((1, Hh, Nn, Dd))).astype(np.float32))
    k = f32_to_bf16_bits((2.0 * rng.standard_normal((1, Hh, Nn, Dd))).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((1, Hh, Nn, Dd)).astype(np.float32))
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    scale = 1 / math.sqrt(Dd)
    out = torch.empty_like(tq)
    att(tq, tk, tv, out, (1, 0), scale)
    torch.cuda.synchronize()
    want = sparse_attention(q, k, v, shared_mask, None, scale, blk, blk)
    assert np.abs(bits_to_f64(from_dev(out)) - want).max() <= MAX_ABS
    serial = out.view(torch.int16).clone()
    # the same key on two streams at once, several rounds
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = [[torch.empty_like(tq) for _ in range(5)] for _ in range(2)]
    torch.cuda.synchronize()
    for r in range(5):
        for si, st in enumerate((s1, s2)):
            outs[si][r].view(torch.int16).fill_(0x7FC1)
            st.wait_stream(torch.cuda.current_stream())
            att(tq, tk, tv, outs[si][r], (2, 0), scale, stream=st.cuda_stream)
    torch.cuda.synchronize()
    for si in range(2):
        for r in range(5):
            assert torch.equal(outs[si][r].view(torch.int16), serial), (si, r)
