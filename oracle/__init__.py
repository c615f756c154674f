"""CPU oracle for block-sparse attention with repeated query blocks, for the
spatial-row anchor scheme, for the calibration steps that produce a mask and for
the skip-list tools of the supplement.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 NumPy written from the paper's
definitions; it shares no code with the HIP library and must never be imported
by the product package.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` use it.

Pin status (see tests/test_oracle_pins.py, tests/test_pattern_oracle.py and
tests/test_anchor_oracle_pins.py, tests/test_calibration_oracle_pins.py, tests/test_skiplist_oracle_pins.py): every function below is pinned by
brute force on tiny inputs, a library routine on a special case, closed forms
and invariants.  No function is "parity unpinned".
"""
from .attention import (  # noqa: F401
    bf16_bits_to_f64,
    expand_block_mask,
    f16_bits_to_f64,
    restricted_softmax_rows,
    sparse_attention,
    sparse_attention_blocks,
    sparse_attention_lse,
)
from .anchor import anchor_attention, anchor_rows, anchor_token_maps, nearest_anchor, spatial_similarity, spatial_similarity_rows  # noqa: F401
from .calibration import block_energy, block_energy_rows, epsilon_schedule, flag_heads, schedule_base_level, schedule_constants, select_blocks, select_row, vote  # noqa: F401
from . import skiplist  # noqa: F401
from .pattern import compile_pattern, pattern_sizes, PatternError  # noqa: F401
