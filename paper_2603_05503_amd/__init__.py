"""Python binding of libcalibatt (block-sparse attention forward for gfx950).

Argument marshalling only: every step of the path runs in the C/HIP library.
torch is used for device buffers and streams.  There is no fallback: if the
library has not been built, loading fails with an error.
"""
from .binding import (  # noqa: F401
    KERNEL_AUTO,
    KERNEL_INTERLEAVED,
    KERNEL_TWO_WORKGROUPS,
    CalibattError,
    DeviceAnchorMap,
    DevicePattern,
    HostAnchorMap,
    HostPattern,
    anchor_attn_fwd,
    anchor_split_plan,
    anchor_map,
    anchor_partner,
    block_energy,
    block_energy_workspace_bytes,
    compile_pattern,
    encode_intervals,
    flag_heads,
    epsilon_schedule,
    library_path,
    load_library,
    merge_intervals,
    pattern_sizes,
    schedule_base_level,
    schedule_constants,
    select_blocks,
    select_blocks_device,
    vote_accumulate_device,
    share_timesteps,
    sparse_attn_fwd,
    spatial_similarity,
    spatial_similarity_static,
    strerror,
    version,
    vote_accumulate,
    vote_finish,
    vote_masks,
)
from .pipeline import CalibAttention, CalibrationResult, Calibrator, load_calibration, save_calibration  # noqa: F401,E402
