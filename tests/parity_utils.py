"""Kept for the tests' imports: the helpers live in workloads/device.py."""
from workloads.device import (  # noqa: F401
    MAX_ABS,
    MEAN_ABS,
    assert_parity,
    assert_repeats_bitwise,
    bits_to_f64,
    error_stats,
    from_dev,
    run_gpu,
    to_dev,
)
