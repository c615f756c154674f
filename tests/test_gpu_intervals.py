"""GPU tests of the interval form of the pattern: the forward must produce the
same bits as with the index form (same kernel arithmetic, same block order) and
stay within tolerance of the oracle."""
import math

import numpy as np
import pytest

from oracle import sparse_attention, sparse_attention_blocks
from tests.parity_utils import MAX_ABS, assert_parity, assert_repeats_bitwise, bits_to_f64, from_dev, to_dev
from workloads import f32_to_bf16_bits, make_workload, random_mask

pytestmark = pytest.mark.gpu


def _qkv(seed, B, H, N, D, gain=1.0):
    rng = np.random.default_rng(seed)
    q = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    k = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    return q, k, v


def _both(lib, q, k, v, hp, scale, persistent=True):
    import torch

    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    outs = []
    for intervals in (False, True):
        dp = hp.to_device(persistent=persistent, intervals=intervals)
        out = torch.empty_like(tq)
        out.view(torch.int16).fill_(0x7FC1)
        lib.sparse_attn_fwd(tq, tk, tv, out, dp, scale)
        torch.cuda.synchronize()
        outs.append(from_dev(out))
    return outs


@pytest.mark.parametrize("B,H,N,D,bq,bk,density,rep", [
    (1, 2, 1024, 64, 64, 64, 0.4, 0.2),
    (2, 3, 1500, 128, 128, 128, 0.3, 0.2),
    (1, 2, 1000, 128, 64, 128, 0.5, 0.0),
    (1, 2, 1000, 64, 128, 64, 0.5, 0.3),
    (1, 1, 700, 128, 128, 128, 0.0, 0.0),   # only the forced diagonal
    (1, 1, 700, 128, 128, 128, 1.0, 0.0),   # one run per row
    (1, 2, 1500, 128, 128, 96, 0.4, 0.2),   # three sub-tiles per key block
    (1, 2, 1500, 128, 128, 160, 0.4, 0.2),  # five
    (1, 2, 1500, 128, 128, 192, 0.4, 0.0),
])
@pytest.mark.parametrize("persistent", [False, True])
def test_intervals_equal_indices(lib, B, H, N, D, bq, bk, density, rep, persistent):
    print(f"intervals B={B} H={H} N={N} D={D} {bq}x{bk} density={density} persistent={persistent}", flush=True)
    q, k, v = _qkv(41 + N + D, B, H, N, D, 2.0)
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask, repeat = random_mask(43, H, nbq, nbk, density, rep, keep_diagonal=True, tail_partial=(N % bq) != 0)
    mask[0, nbq // 2, :] = 0  # an empty row
    hp = lib.compile_pattern(mask, repeat, H, N, bq, bk, 3)
    by_index, by_interval = _both(lib, q, k, v, hp, 1 / math.sqrt(D), persistent)
    assert (by_index == by_interval).all()
    assert_parity(by_interval, sparse_attention(q, k, v, mask, repeat, 1 / math.sqrt(D), bq, bk))
    assert_repeats_bitwise(by_interval, repeat, bq, N)


def test_row_longer_than_one_lds_chunk(lib):
    """More than 2048 kept blocks in a row: the column list is expanded in pieces."""
    print("intervals long row", flush=True)
    B, H, N, D, blk = 1, 1, 140000, 64, 64
    nb = -(-N // blk)  # 2188
    q, k, v = _qkv(47, B, H, N, D, 1.5)
    rng = np.random.default_rng(48)
    mask = np.zeros((H, nb, nb), np.uint8)
    mask[0, np.arange(nb), np.arange(nb)] = 1
    mask[0, 5, :] = 1                                   # one run of 2188 blocks
    mask[0, 9, :] = (rng.random(nb) < 0.97)             # many runs, more than 2048 kept blocks
    mask[0, 9, 2047:2052] = [1, 0, 1, 1, 0]
    mask[0, nb - 1, ::2] = 1                            # the ragged last block, alternating
    assert mask[0, 9].sum() > 2048
    hp = lib.compile_pattern(mask, None, H, N, blk, blk, 1)
    by_index, by_interval = _both(lib, q, k, v, hp, 0.125)
    assert (by_index == by_interval).all()
    items = [(0, 0, 5), (0, 0, 9), (0, 0, nb - 1), (0, 0, 100)]
    want = sparse_attention_blocks(q, k, v, mask, None, 0.125, blk, blk, items)
    for (b, h, r), w in zip(items, want):
        got = bits_to_f64(by_interval[b, h, r * blk : r * blk + w.shape[0]])
        assert np.abs(got - w).max() <= MAX_ABS, r


def test_wan480_interval_pattern(lib):
    """Bench workload in the interval form: same bits as the index form; the index
    lists shrink."""
    print("intervals wan480", flush=True)
    wl = make_workload("wan480", heads=8)
    hp = lib.compile_pattern(wl.mask, wl.repeat, wl.H, wl.N, wl.block_q, wl.block_k, 3)
    by_index, by_interval = _both(lib, wl.q, wl.k, wl.v, hp, wl.scale)
    assert (by_index == by_interval).all()
    a, b = hp.to_device(intervals=False).index_bytes, hp.to_device(intervals=True).index_bytes
    print(f"index bytes {a}, interval bytes {b}", flush=True)
    assert b < a
