"""The forward calls under HIP graph capture: the library launches kernels only
(the persistent scheduler re-arms its own counters, nothing is cleared with a
memset), so a captured graph must replay to the eager result every time."""
import math

import numpy as np
import pytest

from tests.parity_utils import from_dev, to_dev
from workloads import f32_to_bf16_bits, random_mask

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager(lib):
    import torch

    print("graph capture", flush=True)
    B, H, N, D, blk = 4, 8, 4000, 128, 128  # more work items than resident workgroups: persistent launch
    F, Hs, Ws = 5, 10, 80
    rng = np.random.default_rng(17)
    q, k, v = (f32_to_bf16_bits((2.0 * rng.standard_normal((B, H, N, D))).astype(np.float32)) for _ in range(3))
    nb = -(-N // blk)
    mask, repeat = random_mask(18, H - 2, nb, nb, 0.3, 0.2, keep_diagonal=True, tail_partial=True)
    hp = lib.compile_pattern(mask, repeat, H - 2, N, blk, blk, 3)
    dp = hp.to_device(persistent=True, intervals=True, head_map=list(range(2, H)))
    assert hp.n_work * B > 512
    amap = lib.anchor_map(N, F, Hs, Ws, 3).to_device()
    heads = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    scale = 1 / math.sqrt(D)

    def run(out, stream=None):
        lib.sparse_attn_fwd(tq, tk, tv, out, dp, scale, stream=stream)
        lib.anchor_attn_fwd(tq, tk, tv, out, heads, amap, scale, stream=stream)

    eager = torch.empty_like(tq)
    run(eager)  # also the warm-up: kernel attributes are set outside the capture
    torch.cuda.synchronize()
    want = from_dev(eager)
    assert np.isfinite((want.astype(np.uint32) << 16).view(np.float32)).all()

    out = torch.empty_like(tq)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run(out, stream=side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for i in range(4):
        out.view(torch.int16).fill_(0x7FC1)   # eager work between the replays
        run(eager)                            # shares the scheduler workspace with the graph: same stream order
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (from_dev(out) == want).all(), f"replay {i}"
        assert (from_dev(eager) == want).all()


def test_calls_on_two_streams_overlap_safely(lib):
    """No state is shared between calls except the caller's workspaces: two patterns, each with its
    own workspace, launched on two streams at the same time give the bits of the serial runs."""
    import torch

    print("two streams", flush=True)
    B, H, N, D, blk = 2, 16, 3000, 128, 128
    rng = np.random.default_rng(19)
    q, k, v = (f32_to_bf16_bits((2.0 * rng.standard_normal((B, H, N, D))).astype(np.float32)) for _ in range(3))
    nb = -(-N // blk)
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    pats = []
    for seed, dens in ((20, 0.3), (21, 0.6)):
        mask, repeat = random_mask(seed, H, nb, nb, dens, 0.2, keep_diagonal=True, tail_partial=True)
        pats.append(lib.compile_pattern(mask, repeat, H, N, blk, blk, 3).to_device(persistent=True, intervals=seed == 21))
    assert all(dp.host.n_work * B > 512 for dp in pats)
    serial = []
    for dp in pats:
        out = torch.empty_like(tq)
        lib.sparse_attn_fwd(tq, tk, tv, out, dp, 0.09)
        torch.cuda.synchronize()
        serial.append(from_dev(out))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):
        outs = [torch.empty_like(tq) for _ in pats]
        for s in streams:
            s.wait_stream(torch.cuda.current_stream())
        for dp, out, s in zip(pats, outs, streams):
            for _ in range(2):  # back-to-back calls on one stream may share a workspace
                lib.sparse_attn_fwd(tq, tk, tv, out, dp, 0.09, stream=s.cuda_stream)
        torch.cuda.synchronize()
        for out, want in zip(outs, serial):
            assert (from_dev(out) == want).all(), rep


def test_workspace_calls_replay_under_a_graph(lib):
    """The calls that carry a workspace (anchor forward with the key-range split, one-pass block
    energy, selection and vote on the device) launch kernels only and clear nothing with a memset:
    a captured graph of them replays to the eager result, with eager runs on the same workspaces in
    between."""
    import torch

    print("graph capture: workspace calls", flush=True)
    B, H, N, D, blk = 1, 4, 3000, 128, 128
    F, Hs, Ws = 5, 10, 60
    rng = np.random.default_rng(23)
    q, k, v = (f32_to_bf16_bits((2.0 * rng.standard_normal((B, H, N, D))).astype(np.float32)) for _ in range(3))
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    scale = 1 / math.sqrt(D)
    amap = lib.anchor_map(N, F, Hs, Ws, 2).to_device()
    heads = torch.arange(H, dtype=torch.int32, device="cuda")
    n_split, nbytes = lib.anchor_split_plan(B, N, D, H, amap.n_q)
    assert n_split > 1
    ws_anchor = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
    ws_energy = torch.empty(lib.block_energy_workspace_bytes(N, blk, blk) // 4, dtype=torch.float32, device="cuda")
    nb = -(-N // blk)

    def run(out, energy, mask, counts, stream=None):
        lib.anchor_attn_fwd(tq, tk, tv, out, heads, amap, scale, stream=stream, workspace=ws_anchor)
        lib.block_energy(tq, tk, blk, blk, scale, out=energy, stream=stream, workspace=ws_energy)
        lib.select_blocks_device(energy, 0.9, out=mask, stream=stream)
        lib.vote_accumulate_device(mask[0], counts, stream=stream)

    def buffers():
        return (torch.empty_like(tq), torch.empty((B, H, nb, nb), dtype=torch.float32, device="cuda"),
                torch.empty((B, H, nb, nb), dtype=torch.uint8, device="cuda"),
                torch.zeros((H, nb, nb), dtype=torch.int16, device="cuda"))

    eager = buffers()
    run(*eager)  # also the warm-up: kernel attributes are set outside the capture
    torch.cuda.synchronize()
    want_out, want_energy, want_mask = from_dev(eager[0]), eager[1].cpu().numpy(), eager[2].cpu().numpy()
    assert 0 < want_mask.mean() < 1

    graphed = buffers()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run(*graphed, stream=side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for i in range(3):
        graphed[0].view(torch.int16).fill_(0x7FC1)
        graphed[1].fill_(float("nan"))
        ws_anchor.fill_(float("nan"))
        ws_energy.fill_(float("nan"))
        run(*eager)  # eager work on the same workspaces between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert (from_dev(graphed[0]) == want_out).all(), f"replay {i}"
        assert (graphed[1].cpu().numpy() == want_energy).all(), f"replay {i}"
        assert (graphed[2].cpu().numpy() == want_mask).all(), f"replay {i}"
        assert (graphed[3].cpu().numpy().view(np.uint16) == (i + 1) * want_mask[0]).all(), f"replay {i}"
