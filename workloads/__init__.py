"""Seeded synthetic inputs (q/k/v bits, block masks, repeat maps) shared by the
tests, the benchmark and the CPU oracle's callers.

This package holds input *generation* (random draws, bf16 rounding of the drawn
values, mask/repeat-map recipes) and the host/GPU plumbing around a run
(``device.py``).  None of the attention arithmetic and none of the
pattern-compilation logic lives here.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    Geometry,
    Workload,
    bf16_bits_to_f32,
    calibrated_like_mask,
    dictionary_head_masks,
    f32_to_bf16_bits,
    make_qkv,
    make_workload,
    random_mask,
    sweep_pattern,
    tiny_mask,
)
from .device import (  # noqa: F401,E402
    assert_parity,
    assert_repeats_bitwise,
    error_stats,
    from_dev,
    run_gpu,
    to_dev,
)
