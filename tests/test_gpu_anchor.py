"""GPU parity of the spatial-row anchor path (reduced query set + broadcast)
against the fp64 oracle, through the C ABI."""
import math

import numpy as np
import pytest

from oracle import anchor_attention, anchor_token_maps
from tests.parity_utils import MAX_ABS, MEAN_ABS, assert_parity, bits_to_f64, from_dev, to_dev
from workloads import f32_to_bf16_bits

pytestmark = pytest.mark.gpu

POISON = 0x7FC1


def _qkv(seed, B, H, N, D, gain=1.0):
    rng = np.random.default_rng(seed)
    q = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    k = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    return q, k, v


def _run(lib, q, k, v, heads, amap, scale, split=False, expect_split=None):
    """split: through calibatt_anchor_attn_fwd_split with the workspace its plan asks for
    (poisoned with NaN: every value the merge reads must have been written by a part)."""
    import torch

    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    out = torch.empty_like(tq)
    out.view(torch.int16).fill_(POISON)
    hid = torch.tensor(heads, dtype=torch.int32, device="cuda")
    workspace = None
    if split:
        B, H, N, D = q.shape
        n_split, nbytes = lib.anchor_split_plan(B, N, D, len(heads), amap.n_q)
        print(f"  split plan: {n_split} parts, workspace {nbytes} bytes", flush=True)
        if expect_split is not None:
            assert (n_split > 1) == expect_split
        assert (nbytes > 0) == (n_split > 1) and nbytes % 16 == 0
        workspace = torch.full((max(nbytes, 16) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    lib.anchor_attn_fwd(tq, tk, tv, out, hid, amap, scale, workspace=workspace)
    torch.cuda.synchronize()
    return from_dev(out)


# (B, H, heads, F, Hs, Ws, k, extra tokens, D, gain)
CASES = [
    (1, 2, [1], 2, 5, 20, 2, 0, 128, 1.0),       # 200 tokens, 80 computed: a single ragged block
    (2, 3, [2, 0], 3, 7, 20, 3, 37, 128, 2.0),   # 457 tokens, ragged key tail, free tokens, two heads, batch 2
    (1, 2, [0, 1], 4, 6, 33, 1, 0, 64, 2.0),     # head dim 64
    (1, 1, [0], 3, 9, 40, 9, 5, 128, 2.0),       # every row an anchor: plain dense attention
    (1, 9, list(range(9)), 2, 8, 16, 5, 0, 64, 1.0),  # more heads than XCD ranges
]


@pytest.mark.parametrize("split", [False, True], ids=["whole", "split"])
@pytest.mark.parametrize("B,H,heads,F,Hs,Ws,k,extra,D,gain", CASES)
def test_anchor_parity(lib, B, H, heads, F, Hs, Ws, k, extra, D, gain, split):
    print(f"anchor parity B={B} H={H} heads={heads} F={F} Hs={Hs} Ws={Ws} k={k} extra={extra} D={D} split={split}",
          flush=True)
    N = F * Hs * Ws + extra
    q, kk, v = _qkv(21 + F + Hs + Ws + k, B, H, N, D, gain)
    scale = 1 / math.sqrt(D)
    amap = lib.anchor_map(N, F, Hs, Ws, k).to_device()
    # these small shapes fill less than one round of the GPU: every unit is split
    got = _run(lib, q, kk, v, heads, amap, scale, split=split, expect_split=True)
    want = anchor_attention(q, kk, v, heads, F, Hs, Ws, k, scale)
    for i, h in enumerate(heads):
        assert_parity(got[:, h], want[:, i], f"head {h}")
    # heads that are not listed are not touched
    for h in set(range(H)) - set(heads):
        assert (got[:, h] == POISON).all()
    # receivers of one computed query hold the same bits
    q_index, src = anchor_token_maps(N, F, Hs, Ws, k)
    for h in heads:
        assert (got[:, h] == got[:, h][:, q_index[src]]).all()


@pytest.mark.parametrize("split", [False, True], ids=["whole", "split"])
def test_custom_lists_and_invalid_entries_are_safe(lib, split):
    """Lists that do not come from the geometry: rows nobody names stay untouched,
    receivers outside [0, N) are skipped, query indices are clamped, an invalid
    head id is skipped."""
    import torch
    from paper_2603_05503_amd.binding import HostAnchorMap

    print("anchor custom lists", flush=True)
    B, H, N, D = 1, 2, 300, 128
    q, k, v = _qkv(77, B, H, N, D, 2.0)
    q_index = np.array([5, 299, 1000, -3, 17], np.int32)  # 1000 -> 299, -3 -> 0
    dst = [[0, 1, 2], [], [10, -1, 400, 11], [298], [299, 3]]
    dst_ptr = np.concatenate([[0], np.cumsum([len(d) for d in dst])]).astype(np.int32)
    dst_idx = np.array([t for d in dst for t in d], np.int32)
    amap = HostAnchorMap(N=N, n_q=5, q_index=q_index, dst_ptr=dst_ptr, dst_idx=dst_idx).to_device()
    got = _run(lib, q, k, v, [1, 7, -1], amap, 0.09, split=split)
    from oracle.anchor import dense_rows
    from oracle import bf16_bits_to_f64

    qf, kf, vf = (bf16_bits_to_f64(x[0, 1]) for x in (q, k, v))
    rows = dense_rows(qf[[5, 299, 299, 0, 17]], kf, vf, 0.09)
    written = {}
    for i, d in enumerate(dst):
        for t in d:
            if 0 <= t < N:
                written[t] = i
    for t in range(N):
        if t in written:
            diff = np.abs(bits_to_f64(got[0, 1, t]) - rows[written[t]])
            assert diff.max() <= MAX_ABS, t
        else:
            assert (got[0, 1, t] == POISON).all(), t
    assert (got[0, 0] == POISON).all()


@pytest.mark.parametrize("split", [False, True], ids=["whole", "split"])
def test_long_receiver_lists(lib, split):
    """One computed query broadcast to more receivers than one staging chunk holds."""
    from paper_2603_05503_amd.binding import HostAnchorMap

    print("anchor long lists", flush=True)
    B, H, N, D = 1, 1, 5000, 64
    q, k, v = _qkv(78, B, H, N, D)
    q_index = np.array([7, 4000, 123], np.int32)
    dst = [list(range(0, 2500)), list(range(2500, 2501)), list(range(2501, 5000))]
    dst_ptr = np.concatenate([[0], np.cumsum([len(d) for d in dst])]).astype(np.int32)
    dst_idx = np.array([t for d in dst for t in d], np.int32)
    amap = HostAnchorMap(N=N, n_q=3, q_index=q_index, dst_ptr=dst_ptr, dst_idx=dst_idx).to_device()
    got = _run(lib, q, k, v, [0], amap, 0.125, split=split)
    assert (got[0, 0, :2500] == got[0, 0, 0]).all()
    assert (got[0, 0, 2501:] == got[0, 0, 2501]).all()
    from oracle.anchor import dense_rows
    from oracle import bf16_bits_to_f64

    qf, kf, vf = (bf16_bits_to_f64(x[0, 0]) for x in (q, k, v))
    rows = dense_rows(qf[[7, 4000, 123]], kf, vf, 0.125)
    for t, i in ((0, 0), (2499, 0), (2500, 1), (2501, 2), (4999, 2)):
        assert np.abs(bits_to_f64(got[0, 0, t]) - rows[i]).max() <= MAX_ABS


@pytest.mark.parametrize("split", [False, True], ids=["whole", "split"])
def test_wan480_k5_sampled_parity(lib, split):
    """The paper's setting (Wan 480p geometry, k = 5) on a few heads of the full
    shape: sampled computed queries against the oracle, every token bitwise
    against the anchor it copies, a second run bit for bit.  With two heads the
    86 units leave 10-11 per XCD, all in the last round: with `split` each is cut."""
    import torch
    from oracle.anchor import dense_rows
    from oracle import bf16_bits_to_f64

    print("anchor wan480 k=5", flush=True)
    B, H, F, Hs, Ws, k, D = 1, 4, 21, 30, 52, 5, 128
    N = F * Hs * Ws
    q, kk, v = _qkv(79, B, H, N, D, 1.5)
    scale = 1 / math.sqrt(D)
    amap = lib.anchor_map(N, F, Hs, Ws, k).to_device()
    heads = [3, 1]
    got = _run(lib, q, kk, v, heads, amap, scale, split=split, expect_split=True)
    again = _run(lib, q, kk, v, heads, amap, scale, split=split)
    assert (got == again).all()
    q_index, src = anchor_token_maps(N, F, Hs, Ws, k)
    for h in heads:
        assert (got[0, h] == got[0, h][q_index[src]]).all()
    assert (got[0, 0] == POISON).all() and (got[0, 2] == POISON).all()
    rng = np.random.default_rng(5)
    sample = np.unique(np.concatenate([rng.integers(0, q_index.size, 96), [0, q_index.size - 1, 127, 128]]))
    worst, total, n = 0.0, 0.0, 0
    for h in heads:
        qf, kf, vf = (bf16_bits_to_f64(x[0, h]) for x in (q, kk, v))
        want = dense_rows(qf[q_index[sample]], kf, vf, scale)
        d = np.abs(bits_to_f64(got[0, h][q_index[sample]]) - want)
        worst, total, n = max(worst, float(d.max())), total + float(d.sum()), n + d.size
    print(f"max_abs {worst:.3e} mean_abs {total / n:.3e}", flush=True)
    assert worst <= MAX_ABS and total / n <= MEAN_ABS


def test_split_workspace_too_small_is_refused(lib):
    """A workspace shorter than the plan asks for is an error, not a fault."""
    import torch
    from paper_2603_05503_amd.binding import CalibattError

    print("anchor split: short workspace", flush=True)
    B, H, F, Hs, Ws, k, D = 1, 2, 3, 7, 20, 3, 128
    N = F * Hs * Ws
    q, kk, v = _qkv(80, B, H, N, D)
    amap = lib.anchor_map(N, F, Hs, Ws, k).to_device()
    n_split, nbytes = lib.anchor_split_plan(B, N, D, 2, amap.n_q)
    assert n_split > 1 and nbytes > 16
    tq, tk, tv = to_dev(q), to_dev(kk), to_dev(v)
    out = torch.empty_like(tq)
    hid = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    small = torch.empty(nbytes // 4 - 4, dtype=torch.float32, device="cuda")
    with pytest.raises(CalibattError) as e:
        lib.anchor_attn_fwd(tq, tk, tv, out, hid, amap, 0.1, workspace=small)
    assert e.value.status == -7


def test_split_plan_at_the_paper_shapes(lib):
    """Wan 480p, 40 heads (supplement, anchor benchmark): k = 5 leaves 215 units per
    XCD, 23 beyond three full rounds of 64, cut in two; k = 30 (every row) leaves
    none to gain from on a 64-slot XCD only if the plan says so - the plan is
    checked against its own definition here."""
    N, D, H = 21 * 30 * 52, 128, 40
    for k in (1, 2, 3, 4, 5, 10, 15, 30):
        n_q = 21 * k * 52
        n_split, nbytes = lib.anchor_split_plan(1, N, D, H, n_q)
        units = H * -(-n_q // 128)
        rem = max((units * (x + 1) // 8 - units * x // 8) % 64 for x in range(8))
        cost = lambda s: -(-rem * s // 64) / s + 0.01 * s
        best = min(range(1, 9), key=lambda s: (cost(s) if s > 1 else 1.0, s))
        want = best if rem and cost(best) <= 0.9 and best > 1 else 1
        print(f"  k={k}: units {units}, rem {rem}, n_split {n_split}, workspace {nbytes / 2**20:.1f} MiB", flush=True)
        assert n_split == want
        assert nbytes == (8 * rem * n_split * (128 * D + 128) * 4 if n_split > 1 else 0)
