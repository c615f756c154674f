"""GPU property tests: what must hold at any size (no oracle needed), plus the
degenerate cases of the method."""
import math

import numpy as np
import pytest

from oracle import sparse_attention
from tests.parity_utils import assert_parity, assert_repeats_bitwise, bits_to_f64, from_dev, run_gpu, to_dev
from workloads import f32_to_bf16_bits, random_mask

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("kernel_variant")]


def _qkv(seed, B, H, N, D, gain=1.0):
    rng = np.random.default_rng(seed)
    q = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    k = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    return q, k, v


def test_skipped_blocks_are_never_touched(lib):
    """NaN-poisoned K/V in skipped blocks must not change a single output bit."""
    print("poison", flush=True)
    B, H, N, D, blk = 1, 2, 1152, 128, 128
    q, k, v = _qkv(5, B, H, N, D, 2.0)
    nb = N // blk
    mask, repeat = random_mask(6, H, nb, nb, 0.4, 0.0, keep_diagonal=True)
    mask[:, :, 3] = 0  # column block 3 is skipped by every row of every head
    base, _ = run_gpu(lib, q, k, v, mask, repeat, 1 / math.sqrt(D), blk, blk)
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 3 * blk : 4 * blk] = 0x7FC0  # bf16 NaN
    v2[:, :, 3 * blk : 4 * blk] = 0x7FC0
    got, _ = run_gpu(lib, q, k2, v2, mask, repeat, 1 / math.sqrt(D), blk, blk)
    assert np.isfinite(bits_to_f64(got)).all()
    assert (got == base).all()


def test_rows_without_kept_blocks_are_zero(lib):
    print("empty rows", flush=True)
    B, H, N, D, blk = 1, 1, 500, 64, 64
    q, k, v = _qkv(7, B, H, N, D)
    nb = -(-N // blk)
    mask = np.ones((H, nb, nb), np.uint8)
    mask[0, 2, :] = 0
    mask[0, nb - 1, :] = 0  # the ragged last block as well
    got, _ = run_gpu(lib, q, k, v, mask, None, 0.125, blk, blk)
    assert not got[0, 0, 2 * blk : 3 * blk].any()
    assert not got[0, 0, (nb - 1) * blk :].any()
    assert_parity(got, sparse_attention(q, k, v, mask, None, 0.125, blk, blk))


def test_all_rows_repeated_but_one(lib):
    print("fan-out", flush=True)
    B, H, N, D, blk = 2, 1, 700, 128, 128
    q, k, v = _qkv(8, B, H, N, D, 2.0)
    nb = -(-N // blk)
    mask = np.ones((H, nb, nb), np.uint8)
    repeat = np.zeros((H, nb), np.int32)
    repeat[0, 0] = -1  # block 0 computed, every other block (incl. the short last one) copies it
    got, dp = run_gpu(lib, q, k, v, mask, repeat, 0.1, blk, blk)
    assert dp.host.n_work == 1 and dp.host.n_repeat == nb - 1
    assert_repeats_bitwise(got, repeat, blk, N)
    assert_parity(got, sparse_attention(q, k, v, mask, repeat, 0.1, blk, blk))


def test_writes_stay_inside_the_output(lib):
    """Guard rows after the tensor must survive (ragged N, repeats into the tail)."""
    import torch

    print("guard", flush=True)
    B, H, N, D, blk = 1, 2, 333, 64, 64
    q, k, v = _qkv(9, B, H, N, D)
    nb = -(-N // blk)
    mask, repeat = random_mask(10, H, nb, nb, 0.6, 0.4, keep_diagonal=True, tail_partial=True)
    dp = lib.compile_pattern(mask, repeat, H, N, blk, blk, 1).to_device()
    guard = 4096
    buf = torch.full((B * H * N * D + guard,), -7.0, dtype=torch.bfloat16, device="cuda")
    out = buf[: B * H * N * D].view(B, H, N, D)
    lib.sparse_attn_fwd(to_dev(q), to_dev(k), to_dev(v), out, dp, 0.125)
    torch.cuda.synchronize()
    assert (buf[B * H * N * D :] == -7.0).all()
    assert_parity(from_dev(out), sparse_attention(q, k, v, mask, repeat, 0.125, blk, blk))


@pytest.mark.parametrize("persistent", [False, True])
def test_run_to_run_bitwise_and_scheduler_independent(lib, persistent):
    """Same bits on every run, whatever the schedule order or the launch mode
    (kv blocks of a row are always reduced in ascending order)."""
    import torch

    print(f"determinism persistent={persistent}", flush=True)
    B, H, N, D, blk = 1, 8, 4000, 128, 128
    q, k, v = _qkv(11, B, H, N, D, 2.0)
    nb = -(-N // blk)
    mask, repeat = random_mask(12, H, nb, nb, 0.3, 0.2, keep_diagonal=True, tail_partial=True)
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    ref = None
    for order in (0, 1, 2, 3, 4, 1):
        dp = lib.compile_pattern(mask, repeat, H, N, blk, blk, order).to_device(persistent=persistent)
        for _ in range(2):  # the second call also checks that the work counter was re-armed
            out = torch.zeros_like(tq)
            lib.sparse_attn_fwd(tq, tk, tv, out, dp, 0.088)
            torch.cuda.synchronize()
            bits = from_dev(out)
            if ref is None:
                ref = bits
            assert (bits == ref).all(), order
        if persistent:
            words = dp.counter.cpu().tolist()
            assert words[:9] == [0] * 9  # counters re-armed by the last workgroup
            assert words[12:] == [0] * 4  # reserved words untouched
    assert_repeats_bitwise(ref, repeat, blk, N)


@pytest.mark.parametrize("D,blk,N", [(64, 64, 300), (128, 128, 600)])
def test_negative_and_zero_scale(lib, D, blk, N):
    print(f"scale sign D={D} blk={blk}", flush=True)
    B, H = 1, 1
    q, k, v = _qkv(13, B, H, N, D, 2.0)
    nb = -(-N // blk)
    mask, _ = random_mask(14, H, nb, nb, 0.7, keep_diagonal=True)
    for scale in (-0.125, 0.0):
        got, _ = run_gpu(lib, q, k, v, mask, None, scale, blk, blk)
        assert_parity(got, sparse_attention(q, k, v, mask, None, scale, blk, blk), f"scale {scale}")


def test_large_logits_do_not_overflow(lib):
    print("large logits", flush=True)
    B, H, N, D, blk = 1, 1, 512, 128, 128
    q, k, v = _qkv(15, B, H, N, D, 6.0)  # logits of magnitude ~ 36 * sqrt(128) * scale
    mask = np.ones((H, 4, 4), np.uint8)
    got, _ = run_gpu(lib, q, k, v, mask, None, 1.0, blk, blk)  # scale 1: logits in the hundreds
    assert_parity(got, sparse_attention(q, k, v, mask, None, 1.0, blk, blk))
