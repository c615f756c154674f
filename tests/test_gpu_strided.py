"""GPU tests of the strided entry point: [B, N, H, D] tensors and q, k, v as
slices of one fused [B, N, 3, H, D] tensor must give the same bits as packed
[B, H, N, D] copies of the same data, and must not write outside their rows."""
import math

import numpy as np
import pytest

from oracle import sparse_attention
from tests.parity_utils import assert_parity, from_dev, to_dev
from workloads import f32_to_bf16_bits, random_mask

pytestmark = pytest.mark.gpu


def _qkv(seed, B, H, N, D, gain=2.0):
    rng = np.random.default_rng(seed)
    q = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    k = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    return q, k, v


@pytest.mark.parametrize("B,H,N,D,bq,bk", [(2, 3, 900, 128, 128, 128), (1, 4, 777, 64, 64, 64), (1, 2, 1000, 128, 64, 128),
                                             (1, 3, 900, 128, 128, 160)])
@pytest.mark.parametrize("intervals", [False, True])
def test_strided_layouts_equal_packed(lib, B, H, N, D, bq, bk, intervals):
    import torch

    print(f"strided B={B} H={H} N={N} D={D} {bq}x{bk} intervals={intervals}", flush=True)
    q, k, v = _qkv(61 + N, B, H, N, D)
    nbq, nbk = -(-N // bq), -(-N // bk)
    mask, repeat = random_mask(62, H, nbq, nbk, 0.4, 0.2, keep_diagonal=True, tail_partial=(N % bq) != 0)
    hp = lib.compile_pattern(mask, repeat, H, N, bq, bk, 3)
    scale = 1 / math.sqrt(D)
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)

    def run(qq, kk, vv, out):
        dp = hp.to_device(intervals=intervals)
        lib.sparse_attn_fwd(qq, kk, vv, out, dp, scale)
        torch.cuda.synchronize()

    packed = torch.empty_like(tq)
    run(tq, tk, tv, packed)
    assert_parity(from_dev(packed), sparse_attention(q, k, v, mask, repeat, scale, bq, bk))

    # [B, N, H, D] storage, viewed as [B, H, N, D]
    bnhd = [t.transpose(1, 2).contiguous() for t in (tq, tk, tv)]
    out_bnhd = torch.full((B, N, H, D), -7.0, dtype=torch.bfloat16, device="cuda")
    run(*(t.transpose(1, 2) for t in bnhd), out_bnhd.transpose(1, 2))
    assert torch.equal(out_bnhd.transpose(1, 2).contiguous().view(torch.int16), packed.view(torch.int16))

    # fused projection output [B, N, 3, H, D]; the result goes into a padded [B, N, H + 1, D] buffer
    fused = torch.stack([t.transpose(1, 2) for t in (tq, tk, tv)], dim=2).contiguous()
    views = [fused[:, :, i].transpose(1, 2) for i in range(3)]
    assert not views[0].is_contiguous() and views[0].stride(2) == 3 * H * D
    padded = torch.full((B, N, H + 1, D), -7.0, dtype=torch.bfloat16, device="cuda")
    run(*views, padded[:, :, :H].transpose(1, 2))
    assert torch.equal(padded[:, :, :H].transpose(1, 2).contiguous().view(torch.int16), packed.view(torch.int16))
    assert (padded[:, :, H] == -7.0).all()  # the padding head is untouched


def test_strided_argument_checks(lib):
    import torch
    import ctypes as C
    from paper_2603_05503_amd.binding import _CStrides

    print("strided argument checks", flush=True)
    B, H, N, D = 1, 2, 256, 64
    q, k, v = (to_dev(x) for x in _qkv(63, B, H, N, D))
    out = torch.empty_like(q)
    hp = lib.compile_pattern(np.ones((H, 4, 4), np.uint8), None, H, N, 64, 64, 0)
    dp = hp.to_device()
    raw = lib.load_library().calibatt_sparse_attn_fwd_strided
    ok = _CStrides(H * N * D, N * D, D)

    def call(si, so, qp=None):
        return raw(qp or q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, D, 64, 64, C.byref(dp.c), 0.125,
                   C.byref(si) if si else None, C.byref(so) if so else None, None)

    assert call(ok, ok) == 0
    assert call(None, ok) == -1 and call(ok, None) == -1
    assert call(_CStrides(H * N * D, N * D, D - 8), ok) == -2      # rows would overlap
    assert call(_CStrides(H * N * D, N * D + 4, D), ok) == -2      # not a multiple of 8 elements
    assert call(ok, _CStrides(H * N * D, N * D, 1 << 40)) == -2    # beyond 32-bit byte offsets
    assert call(ok, ok, qp=q.data_ptr() + 2) == -2                 # misaligned pointer
    torch.cuda.synchronize()


def test_pattern_over_a_subset_of_heads(lib):
    """head_map: the pattern's heads act on chosen tensor heads, in any order; heads that no entry
    names and entries outside the tensor's heads write nothing."""
    import torch

    print("head map", flush=True)
    B, H, N, D, blk = 2, 5, 600, 128, 128
    q, k, v = _qkv(91, B, H, N, D)
    nb = -(-N // blk)
    chosen = [3, 0, 7, 4]  # pattern head i acts on tensor head chosen[i]; 7 does not exist
    mask, repeat = random_mask(92, len(chosen), nb, nb, 0.5, 0.3, keep_diagonal=True, tail_partial=True)
    hp = lib.compile_pattern(mask, repeat, len(chosen), N, blk, blk, 3)
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    for intervals in (False, True):
        out = torch.empty_like(tq)
        out.view(torch.int16).fill_(0x7FC1)
        lib.sparse_attn_fwd(tq, tk, tv, out, hp.to_device(intervals=intervals, head_map=chosen), 0.09)
        torch.cuda.synchronize()
        got = from_dev(out)
        for i, h in enumerate(chosen):
            if h >= H:
                continue
            want = sparse_attention(q[:, h : h + 1], k[:, h : h + 1], v[:, h : h + 1], mask[i : i + 1],
                                    repeat[i : i + 1], 0.09, blk, blk)
            assert_parity(got[:, h : h + 1], want, f"tensor head {h}")
        for h in (1, 2):
            assert (got[:, h] == 0x7FC1).all()
    # without a head map the head counts must agree
    with pytest.raises(lib.CalibattError) as e:
        lib.sparse_attn_fwd(tq, tk, tv, torch.empty_like(tq), hp.to_device(), 0.09)
    assert e.value.status == -8


def test_both_paths_on_a_fused_projection_tensor(lib):
    """CalibAttention on q, k, v that are slices of one [B, N, 3, H, D] tensor and an output stored as
    [B, N, H, D]: the sparse forward on three heads and the anchor-row forward on the fourth, no
    transposed copies; same bits as with packed tensors."""
    import torch

    print("pipeline strided", flush=True)
    B, H, D, blk = 1, 4, 128, 128
    F, Hs, Ws = 3, 6, 40
    N = F * Hs * Ws
    q, k, v = _qkv(95, B, H, N, D)
    nb = -(-N // blk)
    mask, _ = random_mask(96, H, nb, nb, 0.5, 0.0, keep_diagonal=True, tail_partial=(N % blk) != 0)
    att = lib.CalibAttention(H, N, D, blk, blk, geometry=(F, Hs, Ws), anchors=2)
    att.add("key", mask, repetitive_heads=[2])
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    packed = torch.empty_like(tq)
    att(tq, tk, tv, packed, "key", 0.09)
    fused = torch.stack([t.transpose(1, 2) for t in (tq, tk, tv)], dim=2).contiguous()  # [B, N, 3, H, D]
    out = torch.full((B, N, H, D), -7.0, dtype=torch.bfloat16, device="cuda")
    att(*(fused[:, :, i].transpose(1, 2) for i in range(3)), out.transpose(1, 2), "key", 0.09)
    torch.cuda.synchronize()
    assert torch.equal(out.transpose(1, 2).contiguous().view(torch.int16), packed.view(torch.int16))
