"""GPU parity of the block-energy kernel (Eq. 5) against the fp64 oracle, through
the C ABI, and the calibration chain built on it (Eq. 6, 8-9 -> pattern ->
sparse forward).

Tolerance of the energies: logits come from bf16 products accumulated in fp32
(relative error ~1e-6 of a logit of magnitude <= ~50, i.e. <= 1e-4 absolute in
the exponent), exp2 is the hardware approximation (~1 ulp), sums are fp32 over
<= 128 x N terms in a fixed tree: relative error of an energy <= ~5e-4.  The
test allows 2e-3 relative plus 2e-7 absolute (entries near the fp32 floor)."""
import math

import numpy as np
import pytest

from oracle import block_energy, block_energy_rows, select_blocks, sparse_attention, spatial_similarity, spatial_similarity_rows
from tests.parity_utils import bits_to_f64, from_dev, to_dev
from workloads import f32_to_bf16_bits

pytestmark = pytest.mark.gpu

RTOL, ATOL = 2e-3, 2e-7


def _qk(seed, B, H, N, D, gain=1.0):
    rng = np.random.default_rng(seed)
    q = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    k = f32_to_bf16_bits((gain * rng.standard_normal((B, H, N, D))).astype(np.float32))
    return q, k


CASES = [
    # B, H, N, D, bq, bk, gain, scale
    (1, 2, 300, 64, 64, 64, 1.0, None),      # ragged, odd number of key tiles
    (2, 2, 777, 128, 128, 128, 2.0, None),   # ragged, batch 2
    (1, 1, 1000, 128, 64, 128, 2.0, None),
    (1, 1, 1000, 128, 128, 64, 2.0, None),
    (1, 3, 384, 64, 128, 128, 1.0, None),    # exact multiple, three key tiles
    (1, 1, 50, 128, 128, 128, 1.0, None),    # shorter than one block
    (1, 2, 512, 128, 128, 128, 2.0, -0.1),   # negative scale
    (1, 1, 640, 128, 128, 128, 5.0, 0.25),   # sharp softmax: logits of magnitude ~ 100
    (1, 9, 256, 64, 64, 64, 1.0, None),      # more heads than XCD ranges
]


def _workspace(lib, N, bq, bk, slices=None):
    """Workspace of the one-pass kernel, NaN-filled: what it reads back it must have written.
    slices=None: the recommended size."""
    import torch

    nbytes = lib.block_energy_workspace_bytes(N, bq, bk)
    one = -(-N // bk) * bq * 4
    assert nbytes == 1024 * one
    if slices is not None:
        nbytes = slices * one
    return torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")


# passes: 2 = calibatt_block_energy; 1 = calibatt_block_energy_onepass with the recommended workspace;
# (1, n) = the same with n slices only (n persistent workgroups walk all query blocks)
@pytest.mark.parametrize("passes", [2, 1, (1, 1), (1, 11)], ids=["two-pass", "one-pass", "one-pass-1wg", "one-pass-11wg"])
@pytest.mark.parametrize("B,H,N,D,bq,bk,gain,scale", CASES)
def test_block_energy_parity(lib, B, H, N, D, bq, bk, gain, scale, passes):
    import torch

    print(f"energy parity B={B} H={H} N={N} D={D} bq={bq} bk={bk} gain={gain} scale={scale} passes={passes}", flush=True)
    q, k = _qk(31 + N + D + bq + bk, B, H, N, D, gain)
    scale = 1 / math.sqrt(D) if scale is None else scale
    tq, tk = to_dev(q), to_dev(k)
    ws = None if passes == 2 else _workspace(lib, N, bq, bk, None if passes == 1 else passes[1])
    E = lib.block_energy(tq, tk, bq, bk, scale, workspace=ws)
    torch.cuda.synchronize()
    got = E.cpu().numpy().astype(np.float64)
    want = block_energy(q, k, scale, bq, bk)
    assert got.shape == want.shape
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, want, rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(got.sum(axis=-1), 1.0, rtol=0, atol=2e-4)
    # same bits on a second run into a poisoned buffer
    E2 = torch.full_like(E, float("nan"))
    lib.block_energy(tq, tk, bq, bk, scale, out=E2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(E, E2)


def test_uniform_attention_gives_block_sizes(lib):
    import torch

    print("energy uniform", flush=True)
    N, D, bq, bk = 700, 128, 128, 64
    q = np.zeros((1, 1, N, D), np.uint16)
    _, k = _qk(5, 1, 1, N, D)
    E = lib.block_energy(to_dev(q), to_dev(k), bq, bk, 1.0).cpu().numpy()
    sizes = np.array([min((c + 1) * bk, N) - c * bk for c in range(-(-N // bk))]) / N
    np.testing.assert_allclose(E[0, 0], np.broadcast_to(sizes, E[0, 0].shape), rtol=1e-5)


@pytest.mark.parametrize("passes", [2, 1], ids=["two-pass", "one-pass"])
def test_wan480_sampled_parity(lib, passes):
    """Full Wan-480p sequence length on a few heads with positionally structured
    q, k (the bench workload's recipe): sampled block-rows against the oracle,
    every block-row sums to 1."""
    import torch
    from workloads import make_workload

    print(f"energy wan480 passes={passes}", flush=True)
    wl = make_workload("wan480", heads=3, qk_gain=1.5)
    ws = _workspace(lib, wl.N, wl.block_q, wl.block_k) if passes == 1 else None
    E = lib.block_energy(to_dev(wl.q), to_dev(wl.k), wl.block_q, wl.block_k, wl.scale, workspace=ws)
    torch.cuda.synchronize()
    got = E.cpu().numpy().astype(np.float64)
    assert got.shape == (1, 3, wl.nbq, wl.nbk) and np.isfinite(got).all()
    np.testing.assert_allclose(got.sum(axis=-1), 1.0, rtol=0, atol=2e-4)
    items = [(0, 0, 0), (0, 1, 100), (0, 2, wl.nbq - 1), (0, 1, 17), (0, 2, 200)]
    for (b, h, r), want in zip(items, block_energy_rows(wl.q, wl.k, wl.scale, wl.block_q, wl.block_k, items)):
        np.testing.assert_allclose(got[b, h, r], want, rtol=RTOL, atol=ATOL)


def test_calibration_chain(lib):
    """Energies -> per-prompt selection -> vote -> compiled pattern -> sparse
    forward.  Masks from the GPU energies are checked for validity against the
    oracle's energies (the two may differ where a running sum sits within the
    energy tolerance of the threshold); the sparse output stays close to dense
    attention because the kept blocks carry >= eps of every row's mass."""
    import torch

    print("calibration chain", flush=True)
    B, H, N, D, blk, eps, tol = 1, 2, 1500, 128, 128, 0.9, 2e-3
    nb = -(-N // blk)
    masks = []
    for prompt in range(3):
        q, k = _qk(200 + prompt, B, H, N, D, 2.5)
        E = lib.block_energy(to_dev(q), to_dev(k), blk, blk, 1 / math.sqrt(D)).cpu().numpy()
        m = lib.select_blocks(E, eps)
        Eo = block_energy(q, k, 1 / math.sqrt(D), blk, blk)
        kept = (Eo * m).sum(axis=-1)
        assert (kept >= eps - tol).all()
        lo, hi = select_blocks(Eo, eps - tol).sum(axis=-1), select_blocks(Eo, eps + tol).sum(axis=-1)
        assert (m.sum(axis=-1) >= lo).all() and (m.sum(axis=-1) <= hi).all()
        masks.append(m[0])
    mask = lib.vote_masks(np.stack(masks), 0.5)
    assert mask.shape == (H, nb, nb) and 0 < mask.mean() < 1
    # run the last prompt through the sparse kernel with its own mask: >= eps of the mass kept
    rng = np.random.default_rng(9)
    v = f32_to_bf16_bits(rng.standard_normal((B, H, N, D)).astype(np.float32))
    own = masks[-1]
    dp = lib.compile_pattern(own, None, H, N, blk, blk, 1).to_device()
    out = torch.empty_like(to_dev(q))
    lib.sparse_attn_fwd(to_dev(q), to_dev(k), to_dev(v), out, dp, 1 / math.sqrt(D))
    torch.cuda.synchronize()
    got = bits_to_f64(from_dev(out))
    want_sparse = sparse_attention(q, k, v, own, None, 1 / math.sqrt(D), blk, blk)
    assert np.abs(got - want_sparse).max() <= 2e-2
    dense = sparse_attention(q, k, v, np.ones_like(own), None, 1 / math.sqrt(D), blk, blk)
    rel = np.linalg.norm(got - dense) / np.linalg.norm(dense)
    print(f"density {own.mean():.3f}, rel. L2 distance to dense attention {rel:.3f}", flush=True)
    assert rel < 0.5


# ---------------------------------------------------------------------------
# spatial similarity score (Section 3.3).  Tolerance: the score is a mean of
# ratios of sums of products of probabilities, each with the relative error of
# the energies (<= ~5e-4); 2e-3 absolute on a value in [0, 1].
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("B,H,F,Hs,Ws,k,extra,D,gain,scale", [
    (1, 2, 2, 5, 20, 2, 0, 128, 1.0, None),      # 200 tokens: one ragged block
    (2, 3, 3, 7, 20, 3, 37, 128, 2.0, None),     # tokens without a position, ragged keys, batch 2
    (1, 2, 4, 6, 33, 1, 0, 64, 2.0, None),       # head dim 64, one anchor
    (1, 1, 3, 9, 40, 9, 5, 128, 2.0, None),      # every row an anchor: score 1
    (1, 2, 2, 8, 16, 3, 0, 64, 3.0, -0.2),       # negative scale
])
def test_spatial_similarity_parity(lib, B, H, F, Hs, Ws, k, extra, D, gain, scale):
    import torch

    print(f"similarity B={B} H={H} F={F} Hs={Hs} Ws={Ws} k={k} extra={extra} D={D}", flush=True)
    N = F * Hs * Ws + extra
    q, kk = _qk(71 + F + Hs + Ws + k, B, H, N, D, gain)
    scale = 1 / math.sqrt(D) if scale is None else scale
    partner = torch.from_numpy(lib.anchor_partner(F, Hs, Ws, k)).cuda()
    tq, tk = to_dev(q), to_dev(kk)
    got = lib.spatial_similarity(tq, tk, partner, Ws, scale)
    torch.cuda.synchronize()
    want = spatial_similarity(q, kk, F, Hs, Ws, k, scale)
    np.testing.assert_allclose(got.cpu().numpy().astype(np.float64), want, rtol=0, atol=2e-3)
    if k == Hs:
        np.testing.assert_allclose(got.cpu().numpy(), 1.0, rtol=0, atol=1e-5)
    again = lib.spatial_similarity(tq, tk, partner, Ws, scale)
    torch.cuda.synchronize()
    assert torch.equal(got, again)


def test_spatial_similarity_separates_repetitive_heads(lib):
    """Head 0: queries independent of the spatial row (the premise of Section 3.3)
    -> score 1; head 1: independent random queries -> a low score.  The paper's
    threshold 0.87 separates them."""
    import torch

    print("similarity separation", flush=True)
    F, Hs, Ws, D, k = 3, 10, 26, 128, 5
    N = F * Hs * Ws
    rng = np.random.default_rng(81)
    base = (2.0 * rng.standard_normal((F, 1, Ws, D))).astype(np.float32)
    q0 = np.broadcast_to(base, (F, Hs, Ws, D)).reshape(N, D)
    q1 = (2.0 * rng.standard_normal((N, D))).astype(np.float32)
    q = f32_to_bf16_bits(np.stack([q0, q1])[None])
    kk = f32_to_bf16_bits((2.0 * rng.standard_normal((1, 2, N, D))).astype(np.float32))
    partner = torch.from_numpy(lib.anchor_partner(F, Hs, Ws, k)).cuda()
    s = lib.spatial_similarity(to_dev(q), to_dev(kk), partner, Ws, 1 / math.sqrt(D)).cpu().numpy()[0]
    print("scores", s, flush=True)
    assert s[0] > 0.999 and s[1] < 0.87


def test_spatial_similarity_wan480_sampled(lib):
    """Full Wan-480p geometry (k = 5) on three heads of the bench workload's q, k:
    the cosines of sampled spatial rows, rebuilt from the kernel's per-token
    sums, against the oracle; the score equals the mean of all rows' cosines."""
    import torch
    from workloads import make_workload

    print("similarity wan480", flush=True)
    wl = make_workload("wan480", heads=3, qk_gain=1.5)
    F, Hs, Ws = wl.geometry
    partner = torch.from_numpy(lib.anchor_partner(F, Hs, Ws, 5)).cuda()
    n_tok = partner.numel()
    work = torch.empty((1, 3, n_tok, 3), dtype=torch.float32, device="cuda")
    score = lib.spatial_similarity(to_dev(wl.q), to_dev(wl.k), partner, Ws, wl.scale, workspace=work)
    torch.cuda.synchronize()
    sums = work.cpu().numpy().astype(np.float64).reshape(3, F * Hs, Ws, 3).sum(axis=2)
    cos = sums[..., 0] / np.sqrt(sums[..., 1] * sums[..., 2])            # [head, frame * row]
    np.testing.assert_allclose(score.cpu().numpy()[0], cos.mean(axis=1), rtol=0, atol=1e-5)
    items = [(0, 0, 0, 0), (0, 1, 10, 6), (0, 2, 20, 29), (0, 1, 5, 15), (0, 0, 13, 12)]
    want = spatial_similarity_rows(wl.q, wl.k, F, Hs, Ws, 5, wl.scale, items)
    for (b, h, f, i), w in zip(items, want):
        assert abs(cos[h, f * Hs + i] - w) <= 2e-3, (h, f, i, cos[h, f * Hs + i], w)
    assert abs(cos[1, 5 * Hs + 15] - 1.0) < 1e-5  # row 15 is an anchor: compared with itself


# ---- Eq. 6 and the vote counters on the device ------------------------------------------------------

def _energy_rows(seed, n_rows, nbk):
    """Rows shaped like block energies (non-negative, summing to about 1) with the cases that decide
    the order: exact ties, zeros, negative zeros, one dominant block, a row that never reaches eps."""
    rng = np.random.default_rng(seed)
    e = rng.random((n_rows, nbk)).astype(np.float32) ** 6
    e /= e.sum(axis=1, keepdims=True)
    e = e.astype(np.float32)
    if n_rows > 6 and nbk > 4:
        e[0, :] = np.float32(1.0 / nbk)                 # all equal: columns ascending
        e[1, ::2] = e[1, 1::2][: e[1, ::2].size] if nbk % 2 == 0 else e[1, ::2]   # pairs of equal energies
        e[2, :] = 0.0                                   # never reaches eps: everything kept
        e[2, 1] = -0.0
        e[3, :] = 0.0
        e[3, nbk // 2] = 1.0                            # one block is enough
        e[4, :] *= 0.5                                  # total 0.5 < eps
        e[5, : nbk // 2] = 0.0                          # zeros in front
        e[6, :] = np.float32(1e-30)                     # tiny values: the running sum is fp64
        e[6, nbk - 1] = 0.9
    return e


@pytest.mark.parametrize("n_rows,nbk,eps", [(40, 256, 0.9), (33, 591, 0.84), (17, 350, 0.99), (9, 1, 0.5),
                                            (12, 2, 0.7), (25, 100, 0.0), (7, 4096, 0.95), (10, 257, 1.5)])
def test_select_blocks_device_is_bit_exact(lib, n_rows, nbk, eps):
    """The device selection equals the oracle's (sequential fp64 sum in sorted order) and the host
    routine's, entry by entry."""
    import torch

    print(f"device select n_rows={n_rows} nbk={nbk} eps={eps}", flush=True)
    e = _energy_rows(90 + nbk, n_rows, nbk)
    got = lib.select_blocks_device(torch.from_numpy(e).cuda(), eps)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    want = select_blocks(e, eps)
    assert got.dtype == np.uint8 and got.shape == want.shape
    assert (got == want).all()
    assert (got == lib.select_blocks(e, eps)).all()


def test_select_blocks_device_refuses_what_it_cannot_hold(lib):
    import torch
    from paper_2603_05503_amd.binding import CalibattError

    with pytest.raises(CalibattError) as err:
        lib.select_blocks_device(torch.zeros((2, 4097), dtype=torch.float32, device="cuda"), 0.9)
    assert err.value.status == -3


def test_vote_counters_on_the_device(lib):
    """Counters after several prompts equal the host routine's; a full counter stays full."""
    import torch

    print("device vote counters", flush=True)
    rng = np.random.default_rng(12)
    n = 100_003
    masks = (rng.random((5, n)) < 0.4).astype(np.uint8) * rng.integers(1, 255, (5, n)).astype(np.uint8)
    host = np.zeros(n, np.uint16)
    dev = torch.zeros(n, dtype=torch.int16, device="cuda")
    for m in masks:
        lib.vote_accumulate(m, host)
        lib.vote_accumulate_device(torch.from_numpy(m).cuda(), dev)
    torch.cuda.synchronize()
    assert (dev.cpu().numpy().view(np.uint16) == host).all()
    full = torch.from_numpy(np.array([65535, 65534, 0], np.uint16).view(np.int16)).cuda()
    lib.vote_accumulate_device(torch.tensor([1, 1, 0], dtype=torch.uint8, device="cuda"), full)
    torch.cuda.synchronize()
    assert full.cpu().numpy().view(np.uint16).tolist() == [65535, 65535, 0]


def test_device_chain_equals_host_chain_at_wan480_rows(lib):
    """Energies of two heads at the Wan 480p length: the device selection of all 512 rows equals the
    host selection of the same energies (both bit-exact routines of the same definition)."""
    import torch

    print("device select on kernel energies, N=32760", flush=True)
    B, H, N, D = 1, 2, 32760, 128
    q, k = _qk(404, B, H, N, D, 2.0)
    E = lib.block_energy(to_dev(q), to_dev(k), 128, 128, 1 / math.sqrt(D))
    got = lib.select_blocks_device(E, 0.9)
    torch.cuda.synchronize()
    want = lib.select_blocks(E.cpu().numpy(), 0.9)
    assert (got.cpu().numpy() == want).all()
    assert 0 < want.mean() < 1


def test_onepass_workspace_too_small_is_refused(lib):
    import torch
    from paper_2603_05503_amd.binding import CalibattError

    q, k = _qk(3, 1, 1, 300, 64)
    ws = torch.empty(5 * 64 - 1, dtype=torch.float32, device="cuda")  # one float short of a slice (5 key blocks x 64 rows)
    with pytest.raises(CalibattError) as err:
        lib.block_energy(to_dev(q), to_dev(k), 64, 64, 0.1, workspace=ws)
    assert err.value.status == -7


def test_select_blocks_device_tolerates_nan(lib):
    """Energies that are not numbers have no defined order, but the call still ends and writes a mask
    of zeros and ones (the header's promise); the rows without NaN are unaffected."""
    import torch

    e = _energy_rows(7, 12, 200)
    bad = e.copy()
    bad[3, 17] = np.nan
    bad[8, :] = np.nan
    got = lib.select_blocks_device(torch.from_numpy(bad).cuda(), 0.9)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert set(np.unique(got)) <= {0, 1}
    clean = [r for r in range(12) if r not in (3, 8)]
    assert (got[clean] == select_blocks(e, 0.9)[clean]).all()
