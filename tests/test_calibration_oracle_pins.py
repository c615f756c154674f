"""Pins for the calibration oracle (CPU only): block energy (Eq. 5), energy
selection (Eq. 6), threshold schedule (Eq. 7 with the parameters of supplement
Section A.1), cross-prompt vote (Eq. 8-9)."""
import itertools
import math

import numpy as np
import pytest

from oracle import sparse_attention
from oracle import calibration as cal
from workloads import f32_to_bf16_bits


def _bits(rng, shape, gain=1.0):
    return f32_to_bf16_bits((gain * rng.standard_normal(shape)).astype(np.float32))


def _f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------ Eq. 5
@pytest.mark.parametrize("N,bq,bk", [(12, 4, 4), (13, 4, 3), (9, 2, 5), (7, 8, 8)])
def test_block_energy_brute_force(N, bq, bk):
    rng = np.random.default_rng(N + bq + bk)
    D = 4
    q, k = _bits(rng, (1, 2, N, D), 1.5), _bits(rng, (1, 2, N, D), 1.5)
    E = cal.block_energy(q, k, 0.4, bq, bk)
    qf, kf = _f64(q[0, 1]).tolist(), _f64(k[0, 1]).tolist()
    nbq, nbk = -(-N // bq), -(-N // bk)
    want = [[0.0] * nbk for _ in range(nbq)]
    for i in range(N):
        logits = [0.4 * sum(qf[i][d] * kf[j][d] for d in range(D)) for j in range(N)]
        m = max(logits)
        e = [math.exp(x - m) for x in logits]
        z = sum(e)
        rows_in_block = min((i // bq + 1) * bq, N) - (i // bq) * bq
        for j in range(N):
            want[i // bq][j // bk] += e[j] / z / rows_in_block
    np.testing.assert_allclose(E[0, 1], np.array(want), rtol=1e-12, atol=1e-15)


def test_block_rows_sum_to_one_and_match_the_attention_oracles_probabilities():
    rng = np.random.default_rng(3)
    B, H, N, D, bq, bk = 2, 2, 50, 8, 8, 16
    q, k, v = _bits(rng, (B, H, N, D), 2.0), _bits(rng, (B, H, N, D), 2.0), _bits(rng, (B, H, N, D))
    E = cal.block_energy(q, k, 0.3, bq, bk)
    np.testing.assert_allclose(E.sum(axis=-1), 1.0, rtol=1e-13)
    # the pinned attention oracle's P, summed per block
    _, P = sparse_attention(q, k, v, np.ones((H, 1, 1), np.uint8), None, 0.3, N, N, return_probs=True)
    nbq, nbk = -(-N // bq), -(-N // bk)
    for r in range(nbq):
        for c in range(nbk):
            blk = P[:, :, r * bq : (r + 1) * bq, c * bk : (c + 1) * bk]
            np.testing.assert_allclose(E[:, :, r, c], blk.sum(axis=(2, 3)) / blk.shape[2], rtol=1e-12, atol=1e-15)


def test_selected_rows_equal_the_full_computation():
    rng = np.random.default_rng(6)
    q, k = _bits(rng, (2, 2, 37, 8), 2.0), _bits(rng, (2, 2, 37, 8), 2.0)
    E = cal.block_energy(q, k, 0.3, 8, 5)
    items = [(0, 0, 0), (1, 1, 4), (0, 1, 2)]
    for (b, h, r), e in zip(items, cal.block_energy_rows(q, k, 0.3, 8, 5, items)):
        assert (e == E[b, h, r]).all()


def test_uniform_attention_gives_block_sizes():
    rng = np.random.default_rng(4)
    N, D, bq, bk = 23, 4, 5, 6
    q = np.zeros((1, 1, N, D), np.uint16)
    k = _bits(rng, (1, 1, N, D))
    E = cal.block_energy(q, k, 1.0, bq, bk)
    sizes = np.array([min((c + 1) * bk, N) - c * bk for c in range(-(-N // bk))]) / N
    np.testing.assert_allclose(E[0, 0], np.broadcast_to(sizes, E[0, 0].shape), rtol=1e-13)


def test_one_dominant_key_block():
    """Keys of block 2 are aligned with every query and huge: nearly all mass there."""
    N, D, bq, bk = 16, 4, 4, 4
    q = f32_to_bf16_bits(np.ones((1, 1, N, D), np.float32))
    kk = np.zeros((1, 1, N, D), np.float32)
    kk[0, 0, 8:12] = 8.0
    E = cal.block_energy(q, f32_to_bf16_bits(kk), 1.0, bq, bk)
    assert (E[0, 0, :, 2] > 1 - 1e-12).all()
    # closed form: 4 keys with logit 32 against 12 with logit 0
    np.testing.assert_allclose(E[0, 0, :, 0], 4 / (4 * math.exp(32) + 12), rtol=1e-12)


# ------------------------------------------------------------------ Eq. 6
def _best_subset(e, eps):
    """Exhaustive search: smallest cardinality reaching eps."""
    n = len(e)
    for size in range(1, n + 1):
        best = max(sum(e[i] for i in s) for s in itertools.combinations(range(n), size))
        if best >= eps:
            return size
    return n


@pytest.mark.parametrize("seed", range(25))
def test_selection_is_the_smallest_set(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 9))
    e = rng.dirichlet(np.full(n, 0.4))
    eps = float(rng.choice([0.3, 0.5, 0.84, 0.99, 1.0]))
    keep = cal.select_row(e, eps)
    size = int(keep.sum())
    assert size == _best_subset(e.tolist(), eps) or (e.sum() < eps and size == n)
    # kept blocks are the largest ones
    assert e[keep == 1].min() >= e[keep == 0].max() if 0 < size < n else True
    assert e[keep == 1].sum() >= eps or size == n
    if size > 1:  # dropping the smallest kept block falls below the threshold
        assert e[keep == 1].sum() - e[keep == 1].min() < eps


def test_selection_hand_worked_rows():
    assert cal.select_row([0.1, 0.6, 0.05, 0.25], 0.5).tolist() == [0, 1, 0, 0]
    assert cal.select_row([0.1, 0.6, 0.05, 0.25], 0.84).tolist() == [0, 1, 0, 1]   # 0.6 + 0.25 = 0.85
    assert cal.select_row([0.1, 0.6, 0.05, 0.25], 0.86).tolist() == [1, 1, 0, 1]
    assert cal.select_row([0.1, 0.6, 0.05, 0.25], 1.0).tolist() == [1, 1, 1, 1]
    assert cal.select_row([0.25, 0.25, 0.25, 0.25], 0.5).tolist() == [1, 1, 0, 0]  # ties: lower column first
    assert cal.select_row([0.25, 0.25, 0.25, 0.25], 0.500001).tolist() == [1, 1, 1, 0]
    assert cal.select_row([0.3, 0.3, 0.3], 0.95).tolist() == [1, 1, 1]            # total below the threshold
    assert cal.select_row([1.0], 0.99).tolist() == [1]
    m = cal.select_blocks(np.array([[[0.7, 0.3], [0.2, 0.8]]]), 0.75)
    assert m.tolist() == [[[1, 1], [0, 1]]] and m.dtype == np.uint8


def test_selection_sums_in_fp64_whatever_the_input_dtype():
    e32 = np.array([0.5, 0.25, 0.125, 0.125], np.float32)
    assert cal.select_row(e32, 0.875).tolist() == [1, 1, 1, 0]
    tiny = np.array([1.0] + [2.0 ** -30] * 8, np.float32)  # fp32 running sum would lose the small terms
    assert cal.select_row(tiny, 1.0 + 5 * 2.0 ** -30).sum() == 6


# ------------------------------------------------------------------ Eq. 7
def test_schedule_matches_the_numbers_the_paper_prints():
    # supplement A.1: A(N) = 0.796 + 1.41e-6 N, C = 0.99, k = 16; Section 3.2: eps runs from 0.99 to 0.84 for Wan
    N, T = 32760, 50
    A = cal.schedule_base_level(N)
    assert abs(A - 0.8422) < 5e-5
    eps = [cal.epsilon_schedule(t, T, A, 0.99, 16.0) for t in range(T)]
    assert eps[0] == 0.99
    assert round(eps[-1], 2) == 0.84
    assert all(a > b for a, b in zip(eps, eps[1:]))
    # closed form at t = T/2 and the distilled-model parameters (A = 0.763, C = 0.863, k = 5.64)
    assert abs(eps[25] - (A + (0.99 - A) * math.exp(-8.0))) < 1e-15
    assert abs(cal.epsilon_schedule(2, 4, 0.763, 0.863, 5.64) - (0.763 + 0.1 * math.exp(-2.82))) < 1e-15
    assert cal.epsilon_schedule(0, 4, 0.763, 0.863, 5.64) == 0.863


def test_schedule_constants_of_both_regimes():
    # supplement A.1 prints both parameter sets; the many-step one reproduces the 0.99 -> 0.84 range of Section 3.2
    A, C, k = cal.schedule_constants(0, 32760)
    assert (C, k) == (0.99, 16.0) and A == cal.schedule_base_level(32760)
    assert round(cal.epsilon_schedule(49, 50, A, C, k), 2) == 0.84
    A720, _, _ = cal.schedule_constants(0, 75600)
    assert abs(A720 - (0.796 + 0.106596)) < 1e-12 and A720 > A   # longer sequences keep more energy
    assert cal.schedule_constants(1, 32760) == (0.763, 0.863, 5.64) == cal.schedule_constants(1, 75600)
    # the distilled schedule on 4 steps: starts at C, decays towards A, never below it
    eps = [cal.epsilon_schedule(t, 4, 0.763, 0.863, 5.64) for t in range(4)]
    assert eps[0] == 0.863 and all(a > b > 0.763 for a, b in zip(eps, eps[1:]))
    with pytest.raises(ValueError):
        cal.schedule_constants(2, 100)


# ------------------------------------------------------------------ Section 3.3: flagging of repetitive heads
def test_flag_heads_hand_worked():
    # three prompts, four heads, gamma = 0.87 (the paper's threshold): means 0.9, 0.87, 0.5, 0.88
    scores = [[0.95, 0.87, 0.2, 1.00],
              [0.90, 0.87, 0.9, 0.80],
              [0.85, 0.87, 0.4, 0.84]]
    flags, means = cal.flag_heads(scores, 0.87)
    assert flags.tolist() == [1, 0, 0, 1]          # a mean equal to gamma does not exceed it
    assert np.allclose(means, [0.9, 0.87, 0.5, 0.88], atol=1e-15)
    # one prompt: the score itself decides; the mean is not a vote (one low prompt can sink a head)
    assert cal.flag_heads([[0.871, 0.869]], 0.87)[0].tolist() == [1, 0]
    assert cal.flag_heads([[1.0], [1.0], [0.5]], 0.87)[0].tolist() == [0]
    assert cal.flag_heads([[1.0], [1.0], [0.62]], 0.87)[0].tolist() == [1]


def test_flag_heads_against_numpy_mean():
    rng = np.random.default_rng(5)
    s = rng.uniform(0.5, 1.0, (7, 40))
    flags, means = cal.flag_heads(s, 0.87)
    assert np.allclose(means, s.mean(axis=0), rtol=0, atol=1e-15)
    far = np.abs(s.mean(axis=0) - 0.87) > 1e-12
    assert (flags[far] == (s.mean(axis=0) > 0.87)[far]).all()
    # planted mistakes: threshold compared with >=, mean over heads instead of prompts, max instead of mean
    tie = [[0.87, 0.9], [0.87, 0.8]]
    assert cal.flag_heads(tie, 0.87)[0].tolist() == [0, 0]
    assert (np.array(tie).mean(axis=0) >= 0.87).tolist() == [True, False]            # ">=" would flag head 0
    assert (np.array(tie).max(axis=0) > 0.87).tolist() == [False, True]              # "max" would flag head 1
    assert (np.array(tie).mean(axis=1) > 0.87).tolist() == [True, False]             # wrong axis gives another answer


# ------------------------------------------------------------------ Eq. 8-9
def test_vote_hand_worked():
    masks = np.array([[[1, 1, 0, 0]], [[1, 0, 1, 0]], [[1, 0, 0, 0]], [[1, 1, 2, 0]]], np.uint8)  # 4 prompts
    assert cal.vote(masks, 0.5).tolist() == [[1, 1, 1, 0]]   # 4/4, 2/4, 2/4, 0/4
    assert cal.vote(masks, 0.51).tolist() == [[1, 0, 0, 0]]
    assert cal.vote(masks, 1.0).tolist() == [[1, 0, 0, 0]]
    assert cal.vote(masks, 0.0).tolist() == [[1, 1, 1, 1]]
    assert cal.vote(masks[:1], 0.5).tolist() == masks[0].tolist()


def test_vote_is_monotone_in_rho():
    rng = np.random.default_rng(5)
    masks = (rng.random((7, 3, 4, 4)) < 0.5).astype(np.uint8)
    prev = None
    for rho in (0.0, 0.2, 0.5, 0.8, 1.0):
        m = cal.vote(masks, rho)
        if prev is not None:
            assert (m <= prev).all()
        prev = m
    assert (cal.vote(masks, 1.0) == masks.min(axis=0)).all()
    assert (cal.vote(masks, 1e-9) == masks.max(axis=0)).all()
