"""Pins for the fp64 attention oracle (CPU only).

The paper prints no worked numerical example of an attention output, so the
oracle is pinned by: brute force in pure Python on tiny inputs, a library
routine on the all-ones special case, closed forms, and invariants.  A set of
deliberately wrong oracles ("mutants") must each fail at least one pin.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import (
    bf16_bits_to_f64,
    sparse_attention,
    sparse_attention_blocks,
)
from workloads import f32_to_bf16_bits, random_mask, tiny_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(rng, shape, gain=1.0):
    return f32_to_bf16_bits((gain * rng.standard_normal(shape)).astype(np.float32))


def _case(seed, B, H, N, D, bq, bk, density=0.5, repeat_frac=0.0, gain=1.0):
    rng = np.random.default_rng(seed)
    q, k, v = (_bits(rng, (B, H, N, D), gain if i < 2 else 1.0) for i in range(3))
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask, repeat = random_mask(seed + 1, H, nbq, nbk, density, repeat_frac, tail_partial=(N % bq) != 0)
    return q, k, v, mask, repeat


# ---------------------------------------------------------------------------
# brute force, written independently: scalar loops, math.exp, token-level mask
# ---------------------------------------------------------------------------
def _brute(q, k, v, mask, repeat, scale, bq, bk):
    B, H, N, D = q.shape
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    out = np.zeros((B, H, N, D))
    for b in range(B):
        for h in range(H):
            for i in range(N):
                r = i // bq
                if repeat is not None and repeat[h, r] >= 0:
                    continue
                js = [j for j in range(N) if mask[h, r, j // bk]]
                if not js:
                    continue
                s = [scale * sum(qf[b, h, i, d] * kf[b, h, j, d] for d in range(D)) for j in js]
                mx = max(s)
                e = [math.exp(x - mx) for x in s]
                z = sum(e)
                for d in range(D):
                    out[b, h, i, d] = sum(e[t] * vf[b, h, js[t], d] for t in range(len(js))) / z
            for i in range(N):
                r = i // bq
                if repeat is not None and repeat[h, r] >= 0:
                    out[b, h, i] = out[b, h, repeat[h, r] * bq + (i - r * bq)]
    return out


BRUTE_CASES = [
    # seed, B, H, N, D, bq, bk, density, repeat_frac
    (1, 1, 2, 32, 4, 8, 8, 0.5, 0.25),
    (2, 2, 1, 29, 3, 8, 8, 0.4, 0.25),  # ragged tail
    (3, 1, 2, 30, 5, 4, 8, 0.5, 0.3),  # bq != bk, both ragged
    (4, 1, 1, 24, 2, 8, 4, 0.3, 0.0),  # bq > bk, sparse enough for empty rows
    (5, 1, 3, 17, 4, 16, 16, 0.7, 0.5),
]


def pin_brute_force(oracle):
    for (seed, B, H, N, D, bq, bk, dens, rep) in BRUTE_CASES:
        q, k, v, mask, repeat = _case(seed, B, H, N, D, bq, bk, dens, rep, gain=2.0)
        got = oracle(q, k, v, mask, repeat, 0.37, bq, bk)
        want = _brute(q, k, v, mask, repeat, 0.37, bq, bk)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def pin_all_ones_is_library_sdpa(oracle):
    rng = np.random.default_rng(11)
    B, H, N, D = 2, 3, 100, 16
    q, k, v = (_bits(rng, (B, H, N, D), 1.5) for _ in range(3))
    for (bq, bk) in [(32, 32), (16, 64), (128, 128)]:
        nbq, nbk = -(-N // bq), -(-N // bk)
        mask = np.ones((H, nbq, nbk), dtype=np.uint8)
        scale = 1.0 / math.sqrt(D)
        got = oracle(q, k, v, mask, None, scale, bq, bk)
        tq, tk, tv = (torch.from_numpy(bf16_bits_to_f64(x)) for x in (q, k, v))
        want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale).numpy()
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def pin_rows_sum_to_one(oracle_with_probs):
    q, k, v, mask, repeat = _case(21, 1, 2, 96, 8, 16, 32, 0.5, 0.2)
    mask[:, :, 0] = 1  # no empty rows in this pin
    out, p = oracle_with_probs(q, k, v, mask, repeat, 0.5, 16, 32)
    for h in range(2):
        for r in range(6):
            rows = slice(r * 16, (r + 1) * 16)
            if repeat[h, r] >= 0:
                assert not p[0, h, rows].any()
                continue
            np.testing.assert_allclose(p[0, h, rows].sum(axis=1), 1.0, rtol=0, atol=1e-14)
            # probability mass sits only on kept blocks (block energies of
            # skipped blocks are exactly 0; kept ones sum to 1, Eq. 5)
            blk = p[0, h, rows].reshape(16, 3, 32).sum(axis=2)
            assert (blk[:, mask[h, r] == 0] == 0).all()
            assert (p[0, h, rows] >= 0).all()


def pin_convex_hull(oracle):
    q, k, v, mask, repeat = _case(31, 1, 2, 80, 6, 16, 16, 0.4, 0.0, gain=3.0)
    mask[:, :, 2] = 1
    out = oracle(q, k, v, mask, None, 0.4, 16, 16)
    vf = bf16_bits_to_f64(v)
    for h in range(2):
        for r in range(5):
            vis = np.repeat(mask[h, r] != 0, 16)[:80]
            lo, hi = vf[0, h, vis].min(axis=0), vf[0, h, vis].max(axis=0)
            o = out[0, h, r * 16 : (r + 1) * 16]
            assert (o >= lo - 1e-12).all() and (o <= hi + 1e-12).all()


def pin_key_shift_invariance(oracle):
    # adding one vector t to every key adds q_i.t to every logit of row i and
    # must not change the output; a large t proves the max is subtracted
    rng = np.random.default_rng(41)
    B, H, N, D = 1, 1, 64, 4
    qf = rng.integers(-3, 4, size=(B, H, N, D)).astype(np.float32)
    kf = rng.integers(-3, 4, size=(B, H, N, D)).astype(np.float32)
    t = np.array([64.0, -32.0, 16.0, 128.0], dtype=np.float32)  # exact in bf16 after the add
    q, k, k2, v = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf), f32_to_bf16_bits(kf + t), _bits(rng, (B, H, N, D))
    assert (bf16_bits_to_f64(k2) == (kf + t).astype(np.float64)).all()
    mask, _ = random_mask(42, H, 4, 4, 0.6, keep_diagonal=True)
    a = oracle(q, k, v, mask, None, 1.0, 16, 16)
    b = oracle(q, k2, v, mask, None, 1.0, 16, 16)
    assert np.isfinite(b).all()
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-9)


def pin_closed_forms(oracle):
    rng = np.random.default_rng(51)
    B, H, N, D, bq, bk = 1, 1, 37, 5, 8, 12  # last kv block holds exactly 1 key (36)
    q, k, v = (_bits(rng, (B, H, N, D)) for _ in range(3))
    nbq, nbk = 5, 4
    vf = bf16_bits_to_f64(v)
    # (a) only the last kv block kept -> a single visible key -> output is v[36] exactly
    mask = np.zeros((H, nbq, nbk), dtype=np.uint8)
    mask[:, :, 3] = 1
    out = oracle(q, k, v, mask, None, 0.3, bq, bk)
    assert (out[0, 0] == vf[0, 0, 36][None, :]).all()
    # (b) q = 0 -> uniform attention -> mean of the visible values
    mask = np.zeros((H, nbq, nbk), dtype=np.uint8)
    mask[0, :, 1] = 1
    mask[0, 2, 3] = 1
    out = oracle(np.zeros_like(q), k, v, mask, None, 0.3, bq, bk)
    np.testing.assert_allclose(out[0, 0, 0], vf[0, 0, 12:24].mean(axis=0), atol=1e-14)
    np.testing.assert_allclose(out[0, 0, 16:24], np.broadcast_to(np.concatenate([vf[0, 0, 12:24], vf[0, 0, 36:37]]).mean(axis=0), (8, D)), atol=1e-14)
    # (c) two visible keys -> logistic weight
    N2 = 2
    q2, k2, v2 = (_bits(rng, (1, 1, N2, D)) for _ in range(3))
    out = oracle(q2, k2, v2, np.ones((1, 1, 1), dtype=np.uint8), None, 0.7, 4, 4)
    qf, kf, vf2 = (bf16_bits_to_f64(x)[0, 0] for x in (q2, k2, v2))
    for i in range(2):
        d = 0.7 * (qf[i] @ kf[0] - qf[i] @ kf[1])
        w0 = 1.0 / (1.0 + math.exp(-d))
        np.testing.assert_allclose(out[0, 0, i], w0 * vf2[0] + (1 - w0) * vf2[1], atol=1e-14)
    # (d) a row with no kept block gives zeros
    mask = np.ones((1, 5, 4), dtype=np.uint8)
    mask[0, 3, :] = 0
    out = oracle(q, k, v, mask, None, 0.3, bq, bk)
    assert not out[0, 0, 24:32].any() and out[0, 0, :24].any()


def pin_block_row_independence(oracle):
    q, k, v, mask, _ = _case(61, 1, 1, 64, 4, 16, 16, 0.5)
    mask[0, 1] = [1, 0, 1, 0]
    base = oracle(q, k, v, mask, None, 0.5, 16, 16)
    # (a) other rows of the mask do not matter
    m2 = mask.copy()
    m2[0, 0] = 1 - m2[0, 0]
    m2[0, 3] = 1
    assert (oracle(q, k, v, m2, None, 0.5, 16, 16)[0, 0, 16:32] == base[0, 0, 16:32]).all()
    # (b) keys/values of skipped blocks do not matter
    k2, v2 = k.copy(), v.copy()
    big = f32_to_bf16_bits(np.full((16, 4), 3.0e30, dtype=np.float32))
    for blk in (1, 3):
        k2[0, 0, blk * 16 : (blk + 1) * 16] = big
        v2[0, 0, blk * 16 : (blk + 1) * 16] = big
    assert (oracle(q, k2, v2, mask, None, 0.5, 16, 16)[0, 0, 16:32] == base[0, 0, 16:32]).all()
    # (c) and kept ones do
    m3 = mask.copy()
    m3[0, 1] = [1, 1, 1, 0]
    assert np.abs(oracle(q, k, v, m3, None, 0.5, 16, 16)[0, 0, 16:32] - base[0, 0, 16:32]).max() > 1e-3


def pin_repeat_is_copy(oracle):
    q, k, v, mask, _ = _case(71, 2, 2, 60, 4, 16, 16, 0.6)  # last block has 12 rows
    mask[:, :, 0] = 1
    repeat = np.full((2, 4), -1, dtype=np.int32)
    repeat[0, 2] = 0
    repeat[0, 3] = 1  # short destination <- full source: leading 12 rows
    repeat[1, 0] = 2
    out = oracle(q, k, v, mask, repeat, 0.5, 16, 16)
    plain = oracle(q, k, v, mask, None, 0.5, 16, 16)
    assert (out[:, 0, 32:48] == out[:, 0, 0:16]).all()
    assert (out[:, 0, 48:60] == out[:, 0, 16:28]).all()
    assert (out[:, 1, 0:16] == out[:, 1, 32:48]).all()
    # sources and untouched blocks are what they are without any repeat map
    assert (out[:, 0, 0:32] == plain[:, 0, 0:32]).all()
    assert (out[:, 1, 16:60] == plain[:, 1, 16:60]).all()
    # and a repeated block is really not computed from its own queries
    assert np.abs(out[:, 0, 32:48] - plain[:, 0, 32:48]).max() > 1e-3


PINS_OUT = [
    pin_brute_force,
    pin_all_ones_is_library_sdpa,
    pin_convex_hull,
    pin_key_shift_invariance,
    pin_closed_forms,
    pin_block_row_independence,
    pin_repeat_is_copy,
]


@pytest.mark.parametrize("pin", PINS_OUT, ids=lambda f: f.__name__)
def test_oracle_pin(pin):
    pin(sparse_attention)


def test_oracle_rows_sum_to_one():
    pin_rows_sum_to_one(lambda *a: sparse_attention(*a, return_probs=True))


def test_blocks_variant_matches_full():
    q, k, v, mask, repeat = _case(81, 2, 2, 75, 8, 16, 32, 0.5, 0.3, gain=2.0)
    full = sparse_attention(q, k, v, mask, repeat, 0.35, 16, 32)
    items = [(b, h, r) for b in range(2) for h in range(2) for r in range(5)]
    blocks = sparse_attention_blocks(q, k, v, mask, repeat, 0.35, 16, 32, items)
    for (b, h, r), o in zip(items, blocks):
        assert (o == full[b, h, r * 16 : r * 16 + o.shape[0]]).all()
        assert o.shape[0] == min(16, 75 - r * 16)


def test_tiny_config_mask_recipe():
    mask, repeat = tiny_mask(123, H=2, nb=16)
    for h in range(2):
        for r in range(16):
            assert mask[h, r, r] and mask[h, r, 0]
            if r:
                assert mask[h, r, r - 1]
            if r < 15:
                assert mask[h, r, r + 1]
        rep = np.flatnonzero(repeat[h] >= 0)
        assert rep.size == 2 and (repeat[h, rep] == 0).all() and 0 not in rep


def test_paper_shape_numbers():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_shapes.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, value, _ = [x.strip() for x in line.split("|")]
            vals[name] = int(value)
    assert vals["wan480_frames"] * vals["wan480_rows"] * vals["wan480_cols"] == vals["wan480_tokens"]
    assert vals["wan480_rows"] * vals["wan480_cols"] == vals["wan480_tokens_per_frame"]
    from workloads import CONFIGS

    g = CONFIGS["wan480"]["geom"]
    assert (g.frames, g.rows, g.cols, g.n_tokens) == (21, 30, 52, vals["wan480_tokens"])
    assert CONFIGS["wan720"]["geom"].n_tokens == vals["wan720_tokens"]
    # the printed maximum of 295 intervals is floor(N_B / 2) with N_B = ceil(N / 128):
    # block counts round up, the last block is partial
    nb = -(-vals["wan720_tokens"] // vals["block"])
    assert nb == 591 and nb // 2 == vals["wan720_max_intervals"]
    assert CONFIGS["wan480"]["H"] == vals["heads"] and CONFIGS["wan480"]["D"] == vals["head_dim"]


# ---------------------------------------------------------------------------
# the pins have teeth: plausible mistakes, planted on the CPU, each fail a pin
# ---------------------------------------------------------------------------
def _mut_no_scale(q, k, v, m, r, s, bq, bk):
    return sparse_attention(q, k, v, m, r, 1.0, bq, bk)


def _mut_sign(q, k, v, m, r, s, bq, bk):
    return sparse_attention(q, k, v, m, r, -s, bq, bk)


def _mut_mask_transposed(q, k, v, m, r, s, bq, bk):
    m = np.asarray(m)
    if m.shape[1] == m.shape[2]:
        m = m.transpose(0, 2, 1)
    return sparse_attention(q, k, v, m, r, s, bq, bk)


def _mut_block_k_is_block_q(q, k, v, m, r, s, bq, bk):
    # keys are assigned to kv blocks with the query block size
    N = q.shape[2]
    m = np.asarray(m)
    j = np.minimum(np.arange(N) // bq, m.shape[2] - 1)
    return sparse_attention(q, k, v, m[:, :, j], r, s, bq, 1)


def _mut_repeat_ignored(q, k, v, m, r, s, bq, bk):
    return sparse_attention(q, k, v, m, None, s, bq, bk)


def _mut_kv_swapped(q, k, v, m, r, s, bq, bk):
    return sparse_attention(q, v, k, m, r, s, bq, bk)


def _mut_tail_keys_visible(q, k, v, m, r, s, bq, bk):
    # pads the sequence with zero keys/values that stay visible
    B, H, N, D = q.shape
    pad = (-N) % bk
    if pad == 0 or (N + pad) % bq != 0 and -(-(N + pad) // bq) != -(-N // bq):
        return sparse_attention(q, k, v, m, r, s, bq, bk)
    z = np.zeros((B, H, pad, D), dtype=np.uint16)
    out = sparse_attention(
        np.concatenate([q, z], 2), np.concatenate([k, z], 2), np.concatenate([v, z], 2), m, r, s, bq, bk
    )
    return out[:, :, :N]


def _mut_no_max_subtraction(q, k, v, m, r, s, bq, bk):
    # exp() of raw logits overflows where the definition does not
    qf, kf = bf16_bits_to_f64(q), bf16_bits_to_f64(k)
    with np.errstate(over="ignore", invalid="ignore"):
        if np.exp(np.abs(s) * np.abs(np.einsum("bhid,bhjd->bhij", qf, kf)).max()) == np.inf:
            return np.full(q.shape, np.nan)
    return sparse_attention(q, k, v, m, r, s, bq, bk)


MUTANTS = [
    _mut_no_scale,
    _mut_sign,
    _mut_mask_transposed,
    _mut_block_k_is_block_q,
    _mut_repeat_ignored,
    _mut_kv_swapped,
    _mut_tail_keys_visible,
    _mut_no_max_subtraction,
]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda f: f.__name__)
def test_pins_catch_mutant(mutant):
    failed = []
    for pin in PINS_OUT:
        try:
            pin(mutant)
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"no pin catches {mutant.__name__}"


# ---------------------------------------------------------------------------
# fp16 inputs and the log-sum-exp output
# ---------------------------------------------------------------------------
def test_f16_widening_matches_numpy_for_every_bit_pattern():
    from oracle import f16_bits_to_f64

    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = f16_bits_to_f64(bits)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_f16_inputs_equal_the_same_values_given_as_bf16():
    """Values representable in both formats must give identical results whichever way they come in."""
    rng = np.random.default_rng(21)
    vals = (rng.integers(-8, 9, (1, 2, 24, 8)) / 4.0).astype(np.float32)  # multiples of 1/4: exact in bf16 and fp16
    as_bf16 = f32_to_bf16_bits(vals)
    as_f16 = vals.astype(np.float16).view(np.uint16)
    mask, repeat = random_mask(22, 2, 3, 3, 0.6, 0.3, keep_diagonal=True)
    a = sparse_attention(as_bf16, as_bf16, as_bf16, mask, repeat, 0.3, 8, 8)
    b = sparse_attention(as_f16, as_f16, as_f16, mask, repeat, 0.3, 8, 8, dtype="f16")
    assert np.array_equal(a, b)


def test_lse_brute_force_and_library():
    from oracle import sparse_attention_lse

    rng = np.random.default_rng(23)
    B, H, N, D, bq, bk = 1, 2, 13, 4, 4, 3
    q, k = _bits(rng, (B, H, N, D), 1.5), _bits(rng, (B, H, N, D), 1.5)
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask, repeat = random_mask(24, H, nbq, nbk, 0.5, 0.3, keep_diagonal=True, tail_partial=True)
    mask[0, 1, :] = 0  # a row without kept keys
    got = sparse_attention_lse(q, k, mask, repeat, 0.4, bq, bk)
    qf, kf = bf16_bits_to_f64(q), bf16_bits_to_f64(k)
    for h in range(H):
        for i in range(N):
            r = i // bq
            src = int(repeat[h, r])
            i_src = i if src < 0 else src * bq + (i - r * bq)
            r_src = i_src // bq
            terms = [math.exp(0.4 * float(qf[0, h, i_src] @ kf[0, h, j])) for j in range(N) if mask[h, r_src, j // bk]]
            want = math.log(sum(terms)) if terms else -math.inf
            assert (got[0, h, i] == want) if not terms else abs(got[0, h, i] - want) < 1e-12, (h, i)
    # all-ones mask: torch.logsumexp
    dense = sparse_attention_lse(q, k, np.ones((H, 1, 1), np.uint8), None, 0.4, N, N)
    ref = torch.logsumexp(0.4 * torch.from_numpy(qf) @ torch.from_numpy(kf).transpose(-1, -2), dim=-1).numpy()
    np.testing.assert_allclose(dense, ref, rtol=1e-13)


def test_lse_merges_results_over_disjoint_key_sets():
    """Outputs over two disjoint masks, weighted by exp(lse), give the output over their union."""
    from oracle import sparse_attention_lse

    rng = np.random.default_rng(25)
    B, H, N, D, blk = 1, 1, 24, 4, 4
    q, k, v = (_bits(rng, (B, H, N, D), 1.5) for _ in range(3))
    nb = N // blk
    m1 = (rng.random((H, nb, nb)) < 0.5).astype(np.uint8)
    m2 = ((rng.random((H, nb, nb)) < 0.5) & (m1 == 0)).astype(np.uint8)
    m1[:, :, 0] = 1
    m2[:, :, 0] = 0
    m2[:, :, 1] = 1
    m1[:, :, 1] = 0
    o1, o2 = (sparse_attention(q, k, v, m, None, 0.5, blk, blk) for m in (m1, m2))
    l1, l2 = (sparse_attention_lse(q, k, m, None, 0.5, blk, blk) for m in (m1, m2))
    w1, w2 = np.exp(l1)[..., None], np.exp(l2)[..., None]
    merged = (w1 * o1 + w2 * o2) / (w1 + w2)
    union = sparse_attention(q, k, v, m1 | m2, None, 0.5, blk, blk)
    np.testing.assert_allclose(merged, union, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(np.log(np.exp(l1) + np.exp(l2)), sparse_attention_lse(q, k, m1 | m2, None, 0.5, blk, blk), rtol=1e-13)
