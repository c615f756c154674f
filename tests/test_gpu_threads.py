"""The forward called from several host threads at once, each on its own stream with its own
scheduler workspace, reproduces the bits of serial calls (the library keeps no state between calls
except per-device launch facts cached through atomics)."""
import threading

import numpy as np
import pytest

from tests.test_gpu_parity import _qkv
from workloads import random_mask, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kernel", ["auto", "2wg"])
def test_four_threads_four_streams(lib, kernel):
    import torch

    from paper_2603_05503_amd import binding

    print(f"threads kernel={kernel}", flush=True)
    which = binding.KERNEL_AUTO if kernel == "auto" else binding.KERNEL_TWO_WORKGROUPS
    B, H, N, D, blk = 1, 6, 128 * 24 + 50, 128, 128
    nb = -(-N // blk)
    n_threads, rounds = 4, 6
    cases = []
    for i in range(n_threads):
        q, k, v = _qkv(700 + i, B, H, N, D, 2.0)
        mask, repeat = random_mask(800 + i, H, nb, nb, 0.3 + 0.1 * i, 0.2, tail_partial=True)
        hp = lib.compile_pattern(mask, repeat, H, N, blk, blk, 4)
        cases.append((to_dev(q), to_dev(k), to_dev(v), hp))
    # serial reference bits, each case with a workspace of its own
    want = []
    for tq, tk, tv, hp in cases:
        out = torch.empty_like(tq)
        lib.sparse_attn_fwd(tq, tk, tv, out, hp.to_device(), 0.09, kernel=which)
        torch.cuda.synchronize()
        want.append(out.view(torch.int16).clone())
    errors = []
    barrier = threading.Barrier(n_threads)

    def worker(i):
        try:
            tq, tk, tv, hp = cases[i]
            stream = torch.cuda.Stream()
            dp = hp.to_device()  # own index tensors and own work counters
            outs = [torch.empty_like(tq) for _ in range(rounds)]
            torch.cuda.synchronize()
            barrier.wait()
            for r in range(rounds):
                outs[r].view(torch.int16).fill_(0x7FC1)
                stream.wait_stream(torch.cuda.current_stream())
                lib.sparse_attn_fwd(tq, tk, tv, outs[r], dp, 0.09, stream=stream.cuda_stream, kernel=which)
            stream.synchronize()
            for r in range(rounds):
                if not torch.equal(outs[r].view(torch.int16), want[i]):
                    errors.append((i, r, "bits differ from the serial call"))
        except Exception as e:  # noqa: BLE001
            errors.append((i, -1, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
