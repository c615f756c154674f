"""GPU parity of the fp16 element type and of the log-sum-exp output against the
fp64 oracle, through calibatt_sparse_attn_fwd_ex.

LSE tolerance: the kernel's row sum adds probabilities rounded to the element
type (relative error <= 2^-9 each for bf16, averaging down over a row) on top of
fp32 logits (absolute error ~1e-5 at these magnitudes) and the hardware log2:
|lse - oracle| <= 5e-3 is several times the worst case."""
import math

import numpy as np
import pytest

from oracle import sparse_attention, sparse_attention_lse
from tests.parity_utils import MAX_ABS, MEAN_ABS, from_dev, to_dev
from workloads import f32_to_bf16_bits, random_mask

pytestmark = pytest.mark.gpu

LSE_ATOL = 5e-3


def _inputs(seed, B, H, N, D, dtype, gain=2.0):
    rng = np.random.default_rng(seed)
    vals = [(gain * rng.standard_normal((B, H, N, D))).astype(np.float32) for _ in range(2)]
    vals.append(rng.standard_normal((B, H, N, D)).astype(np.float32))
    if dtype == "bf16":
        return [f32_to_bf16_bits(x) for x in vals]
    return [x.astype(np.float16).view(np.uint16) for x in vals]


def _dev(bits, dtype):
    import torch

    t = torch.from_numpy(bits.view(np.int16)).cuda()
    return t.view(torch.bfloat16 if dtype == "bf16" else torch.float16)


def _f64(bits, dtype):
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.view(np.float16).astype(np.float64)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,H,N,D,bq,bk,intervals", [
    (1, 2, 1024, 64, 64, 64, False),
    (2, 3, 1500, 128, 128, 128, True),
    (1, 2, 1000, 128, 64, 128, False),
    (1, 2, 777, 64, 128, 64, True),
    (1, 2, 1100, 128, 128, 96, True),     # key blocks of three / five sub-tiles
    (2, 2, 1100, 128, 128, 160, False),
    (1, 2, 1100, 128, 128, 192, True),
])
def test_dtype_and_lse_parity(lib, dtype, B, H, N, D, bq, bk, intervals):
    import torch

    print(f"ex dtype={dtype} B={B} H={H} N={N} D={D} {bq}x{bk} intervals={intervals}", flush=True)
    q, k, v = _inputs(101 + N + D, B, H, N, D, dtype)
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask, repeat = random_mask(102, H, nbq, nbk, 0.4, 0.2, keep_diagonal=True, tail_partial=(N % bq) != 0)
    mask[0, nbq // 2, :] = 0  # a row that keeps nothing: output 0, lse -inf
    repeat[0, nbq // 2] = -1
    repeat[0][repeat[0] == nbq // 2] = -1
    scale = 1 / math.sqrt(D)
    dp = lib.compile_pattern(mask, repeat, H, N, bq, bk, 3).to_device(intervals=intervals)
    tq, tk, tv = (_dev(x, dtype) for x in (q, k, v))
    out = torch.empty_like(tq)
    out.view(torch.int16).fill_(0x7E01 if dtype == "f16" else 0x7FC1)  # NaN patterns
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    lib.sparse_attn_fwd(tq, tk, tv, out, dp, scale, lse=lse)
    torch.cuda.synchronize()
    got = _f64(from_dev(out), dtype)
    want = sparse_attention(q, k, v, mask, repeat, scale, bq, bk, dtype=dtype)
    assert np.isfinite(got).all()
    d = np.abs(got - want)
    assert d.max() <= MAX_ABS and d.mean() <= MEAN_ABS, (d.max(), d.mean())
    got_lse = lse.cpu().numpy().astype(np.float64)
    want_lse = sparse_attention_lse(q, k, mask, repeat, scale, bq, bk, dtype=dtype)
    empty = np.isneginf(want_lse)
    assert empty.any() and np.array_equal(np.isneginf(got_lse), empty)
    assert np.abs(got_lse[~empty] - want_lse[~empty]).max() <= LSE_ATOL
    # the same call without lse gives the same output bits
    out2 = torch.empty_like(tq)
    lib.sparse_attn_fwd(tq, tk, tv, out2, dp, scale)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


def test_lse_merges_two_gpu_results(lib):
    """Two launches over disjoint halves of the key blocks, merged with their LSE, against one launch
    over all of them (what a key-sharded deployment would do)."""
    import torch

    print("ex merge", flush=True)
    B, H, N, D, blk = 1, 2, 1024, 128, 128
    q, k, v = _inputs(111, B, H, N, D, "bf16")
    nb = N // blk
    full = np.ones((H, nb, nb), np.uint8)
    left, right = full.copy(), full.copy()
    left[:, :, nb // 2 :] = 0
    right[:, :, : nb // 2] = 0
    tq, tk, tv = (_dev(x, "bf16") for x in (q, k, v))
    res = []
    for m in (left, right, full):
        dp = lib.compile_pattern(m, None, H, N, blk, blk, 1).to_device()
        out = torch.empty_like(tq)
        lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
        lib.sparse_attn_fwd(tq, tk, tv, out, dp, 0.09, lse=lse)
        res.append((out.float(), lse))
    torch.cuda.synchronize()
    (o1, l1), (o2, l2), (o, l) = res
    w1, w2 = torch.exp(l1 - l).unsqueeze(-1), torch.exp(l2 - l).unsqueeze(-1)
    merged = w1 * o1 + w2 * o2
    # o1, o2 and o are each rounded to bf16 (relative half-ulp 2^-9): the merge of two rounded results can
    # differ from the rounded full result by the kernel's own tolerance plus those three roundings,
    # 2^-9 (w1 |o1| + w2 |o2| + |o|) <= about 2^-8 |o| for outputs that do not cancel.
    assert ((merged - o).abs() <= MAX_ABS + 2.0 ** -8 * o.abs()).all().item()
    assert (torch.logaddexp(l1, l2) - l).abs().max().item() <= LSE_ATOL


def test_ex_argument_checks(lib):
    import ctypes as C
    import torch
    from paper_2603_05503_amd.binding import _CFwdOptions

    print("ex argument checks", flush=True)
    B, H, N, D = 1, 1, 256, 64
    q, k, v = (_dev(x, "bf16") for x in _inputs(121, B, H, N, D, "bf16"))
    out = torch.empty_like(q)
    dp = lib.compile_pattern(np.ones((H, 4, 4), np.uint8), None, H, N, 64, 64, 0).to_device()
    raw = lib.load_library().calibatt_sparse_attn_fwd_ex

    def call(opt):
        return raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, D, 64, 64, C.byref(dp.c), 0.125,
                   C.byref(opt) if opt is not None else None, None)

    assert call(_CFwdOptions(None, None, 0, None)) == 0
    assert call(None) == -1
    assert call(_CFwdOptions(None, None, 2, None)) == -3
    lse = torch.empty(B * H * N + 1, dtype=torch.float32, device="cuda")
    assert call(_CFwdOptions(None, None, 0, lse.data_ptr() + 2)) == -2
    torch.cuda.synchronize()
