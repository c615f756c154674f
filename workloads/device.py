"""Plumbing shared by the GPU tests, the benchmark and the smoke test: move the seeded bf16 bit
patterns to and from the GPU, run the forward through the binding, and compare two arrays against the
tolerance of the benchmark spec.  No attention arithmetic and no pattern logic lives here."""
import numpy as np


def to_dev(bits):
    import torch

    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def from_dev(t):
    """bf16 CUDA tensor -> uint16 bits on the host."""
    import torch

    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def run_gpu(pkg, q, k, v, mask, repeat, scale, bq, bk, order=1, poison_out=True):
    """Returns (out_bits uint16 [B,H,N,D], DevicePattern)."""
    import torch

    B, H, N, D = q.shape
    hp = pkg.compile_pattern(mask, repeat, H, N, bq, bk, order)
    dp = hp.to_device()
    tq, tk, tv = to_dev(q), to_dev(k), to_dev(v)
    out = torch.empty_like(tq)
    if poison_out:
        out.view(torch.int16).fill_(0x7FC1)  # NaN pattern: every row must be overwritten
    pkg.sparse_attn_fwd(tq, tk, tv, out, dp, scale)
    torch.cuda.synchronize()
    return from_dev(out), dp


def bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def error_stats(got_bits, want_f64):
    got = bits_to_f64(got_bits)
    diff = np.abs(got - want_f64)
    denom = np.sqrt((want_f64 ** 2).sum())
    return dict(
        max_abs=float(diff.max()) if diff.size else 0.0,
        mean_abs=float(diff.mean()) if diff.size else 0.0,
        rel_l2=float(np.sqrt((diff ** 2).sum()) / denom) if denom > 0 else 0.0,
        mean_abs_ref=float(np.abs(want_f64).mean()) if diff.size else 0.0,
        finite=bool(np.isfinite(got).all()),
    )


# spec tolerance for bf16 inputs
MAX_ABS = 2e-2
MEAN_ABS = 2e-3


def assert_parity(got_bits, want_f64, what=""):
    st = error_stats(got_bits, want_f64)
    assert st["finite"], (what, st)
    assert st["max_abs"] <= MAX_ABS and st["mean_abs"] <= MEAN_ABS, (what, st)
    return st


def assert_repeats_bitwise(out_bits, repeat, bq, N):
    H, nbq = repeat.shape
    for h in range(H):
        for r in range(nbq):
            s = int(repeat[h, r])
            if s < 0:
                continue
            n = min((r + 1) * bq, N) - r * bq
            assert (out_bits[:, h, r * bq : r * bq + n] == out_bits[:, h, s * bq : s * bq + n]).all(), (h, r, s)
