"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element
by element, on seeded inputs spanning several tiles and ragged tails."""
import math

import numpy as np
import pytest

from oracle import sparse_attention
from tests.parity_utils import assert_parity, assert_repeats_bitwise, error_stats, run_gpu
from workloads import f32_to_bf16_bits, make_workload, random_mask

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("kernel_variant")]


def _qkv(seed, B, H, N, D, gain=1.0):
    rng = np.random.default_rng(seed)
    q = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    k = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    return q, k, v


@pytest.mark.parametrize("gain", [1.0, 2.5])
def test_tiny_config(lib, gain):
    wl = make_workload("tiny", qk_gain=gain)
    print(f"tiny gain={gain}", flush=True)
    got, _ = run_gpu(lib, wl.q, wl.k, wl.v, wl.mask, wl.repeat, wl.scale, wl.block_q, wl.block_k)
    want = sparse_attention(wl.q, wl.k, wl.v, wl.mask, wl.repeat, wl.scale, wl.block_q, wl.block_k)
    st = assert_parity(got, want, "tiny")
    print(st, flush=True)
    assert_repeats_bitwise(got, wl.repeat, wl.block_q, wl.N)
    assert st["rel_l2"] < 1.5e-2


CASES = [
    # D, bq, bk, B, H, N, density, repeat_frac, gain
    (128, 128, 128, 1, 2, 1000, 0.5, 0.25, 2.0),   # ragged tail, 8 blocks
    (128, 128, 128, 2, 1, 640, 0.4, 0.2, 1.0),     # batch 2, exact multiple
    (128, 128, 64, 1, 2, 700, 0.5, 0.2, 2.0),
    (128, 64, 128, 1, 2, 700, 0.5, 0.2, 2.0),
    (128, 64, 64, 1, 1, 500, 0.6, 0.25, 1.0),
    (64, 128, 128, 1, 2, 900, 0.5, 0.25, 2.0),
    (64, 128, 64, 1, 1, 530, 0.5, 0.2, 1.0),
    (64, 64, 128, 1, 1, 530, 0.5, 0.2, 2.0),
    (64, 64, 64, 2, 2, 333, 0.5, 0.3, 2.0),
    (128, 128, 128, 1, 1, 1, 1.0, 0.0, 1.0),       # a single token
    (128, 128, 128, 1, 1, 129, 1.0, 0.0, 1.0),     # tail block of one row / one key
    # key blocks of 96, 160 and 192 keys (three or five sub-tiles per block; an odd total is padded)
    (128, 128, 96, 1, 2, 1000, 0.5, 0.25, 2.0),
    (128, 128, 160, 1, 2, 1111, 0.5, 0.2, 2.0),
    (128, 128, 192, 1, 2, 1000, 0.5, 0.25, 2.0),
    (128, 128, 192, 2, 1, 777, 0.35, 0.0, 1.0),
    (128, 128, 96, 1, 1, 96 * 70 + 5, 1.0, 0.0, 1.0),   # 71 kept blocks in a row: the cached column list is refilled
    (128, 128, 160, 1, 1, 97, 1.0, 0.0, 1.0),           # one short block
    (128, 128, 192, 1, 1, 1, 1.0, 0.0, 1.0),
]


@pytest.mark.parametrize("D,bq,bk,B,H,N,dens,rep,gain", CASES)
def test_random_masks(lib, D, bq, bk, B, H, N, dens, rep, gain):
    print(f"case D={D} bq={bq} bk={bk} B={B} H={H} N={N}", flush=True)
    seed = D + 3 * bq + 7 * bk + N
    q, k, v = _qkv(seed, B, H, N, D, gain)
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask, repeat = random_mask(seed + 1, H, nbq, nbk, dens, rep, tail_partial=(N % bq) != 0)
    scale = 1.0 / math.sqrt(D)
    for order in (0, 1, 2, 3, 4):
        got, _ = run_gpu(lib, q, k, v, mask, repeat, scale, bq, bk, order=order)
        want = sparse_attention(q, k, v, mask, repeat, scale, bq, bk)
        st = assert_parity(got, want, f"order {order}")
        assert_repeats_bitwise(got, repeat, bq, N)
    print(st, flush=True)


@pytest.mark.parametrize("bk", [96, 160, 192])
def test_wide_key_blocks_only_in_the_interleaved_kernel(lib, bk):
    """The two-workgroup kernel is built for key blocks of 64 and 128 keys: asked for by name with
    another width it refuses, it does not fall back."""
    import torch

    from paper_2603_05503_amd import binding
    from tests.parity_utils import to_dev

    print(f"bk={bk} forced two-workgroup kernel", flush=True)
    N, H, D = 500, 1, 128
    q, k, v = _qkv(5, 1, H, N, D)
    mask = np.ones((H, -(-N // 128), -(-N // bk)), np.uint8)
    dp = lib.compile_pattern(mask, None, H, N, 128, bk, 4).to_device()
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    out = torch.empty_like(tq)
    with pytest.raises(binding.CalibattError) as e:
        binding.sparse_attn_fwd(tq, tk, tv, out, dp, 0.1, kernel=binding.KERNEL_TWO_WORKGROUPS)
    assert e.value.status == -3


def test_interleaved_kernel_by_name_is_the_default(lib):
    import torch

    from paper_2603_05503_amd import binding
    from tests.parity_utils import from_dev, to_dev

    print("kernel by name", flush=True)
    N, H, D = 900, 2, 128
    q, k, v = _qkv(6, 1, H, N, D, 2.0)
    mask, repeat = random_mask(7, H, -(-N // 128), -(-N // 128), 0.5, 0.2, tail_partial=True)
    dp = lib.compile_pattern(mask, repeat, H, N, 128, 128, 4).to_device()
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    outs = []
    for kern in (binding.KERNEL_AUTO, binding.KERNEL_INTERLEAVED):
        out = torch.empty_like(tq)
        binding.sparse_attn_fwd(tq, tk, tv, out, dp, 0.1, kernel=kern)
        torch.cuda.synchronize()
        outs.append(from_dev(out))
    assert (outs[0] == outs[1]).all()
