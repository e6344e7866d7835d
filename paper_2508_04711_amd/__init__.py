"""MI355X (gfx950) jagged HSTU attention: thin Python binding over the C-ABI HIP library.

Everything is computed by the HIP kernels in csrc/; this package only marshals arguments.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    HSTU_FLAG_BIAS_PER_PAIR,
    HSTU_FLAG_DKDV_ONE_WAVE,
    HSTU_FLAG_FWD_TILE_128,
    HSTU_FLAG_FWD_TILE_256,
    HSTU_FLAG_NO_PACK,
    HSTU_FLAG_NO_SPLIT,
    HSTU_FLAG_PACK_SHORT,
    HstuError,
    flags,
    hstu_attn_status_string,
    hstu_cp_reorder,
    hstu_cp_ring_pass,
    hstu_cp_ring_pass_bias,
    hstu_debug_dq_atomic_rate,
    hstu_debug_dump_schedule,
    hstu_debug_mfma_loop,
    hstu_debug_timing_begin,
    hstu_debug_timing_end,
    hstu_jagged_attn_bias_bwd,
    hstu_jagged_attn_bias_fwd,
    hstu_jagged_attn_bias_workspace_bytes,
    hstu_jagged_attn_bwd,
    hstu_jagged_attn_cp_partial,
    hstu_jagged_attn_cp_partial_bias,
    hstu_jagged_attn_fwd,
    hstu_jagged_attn_fwd_static,
    hstu_jagged_attn_workspace_bytes,
    hstu_schedule_tile_rows,
    hstu_static_scratch_bytes,
    hstu_validate_offsets_host,
    library_path,
    load_library,
)
