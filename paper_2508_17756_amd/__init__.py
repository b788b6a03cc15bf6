"""MI355X-native tile-denoising hot path: Python binding over libsupergen_tile.so."""
from .binding import (  # noqa: F401
    SG_F32, SG_BF16, SG_OK, SG_ERR_INVALID_ARG, SG_ERR_UNSUPPORTED, SG_ERR_WORKSPACE, SG_ERR_HIP,
    SgError, sg_problem, sg_step_io, load_library, library_path, make_problem,
    sg_version, sg_status_string, sg_problem_validate, sg_workspace_bytes,
    sg_tile_attention, sg_tile_blend, sg_cache_gate, sg_denoise_step_tiled,
    sg_gain_state, sg_gain_step_io, GainState, sg_gain_gate, sg_gain_refresh, sg_denoise_step_gain,
    SG_REGION_MAXMIN, SG_REGION_TOPSELECT, sg_tile_std, sg_region_thresholds,
    sg_tile_blend_update, sg_tile_slice, sg_shift_schedule, sg_partition_tiles, sg_region_control, sg_scheduler_update,
    sg_cache_gate_static, SG_STATIC_GATE_MAX_TILES, sg_tile_similarity,
)
