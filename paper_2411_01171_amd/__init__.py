"""Streamlined-Inference hot path on MI355X: Python binding of the C-ABI library.

Argument marshalling only; every step of the path runs in the HIP kernels of
libsi.so.  There is no CPU fallback: if the library is missing, importing the
binding's entry points raises.
"""
from .binding import (  # noqa: F401
    SI_F32, SI_BF16, SI_BLOCK_TEMPORAL, SI_BLOCK_SPATIAL, SI_AXIS_F, SI_AXIS_HW,
    SiError, lib, library_path, BlockWeights, RehashCache, ResBlockWeights,
    si_resblock_workspace_bytes, si_resblock_live_activation_bytes, si_resblock_forward,
    SI_RESAMPLE_DOWN, SI_RESAMPLE_UP, si_resample_workspace_bytes, si_resample_forward,
    si_workspace_bytes, si_live_activation_bytes, si_windows_in_flight, si_block_forward, si_block_forward_rehash,
    si_block_forward_ex, SI_FWD_WEIGHTS_PACKED,
    si_rehash_scratch_bytes, si_rehash_check, si_rehash_check_sync, si_key_step_search,
    si_init_device, si_rehash_check_static,
    si_stage_timing_enable, si_stage_timing_read, si_status_str, si_abi_version,
)
