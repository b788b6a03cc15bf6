"""fp64 CPU oracle for the tile-based denoising hot path (TEST INFRASTRUCTURE ONLY).

This package is the slow, plain definition of what the HIP kernels compute.  It
shares no code with the HIP path and must never be imported by the product
package: only tests, the smoke check and the CPU-baseline leg of the benchmark
may call it.
"""
from .tile_oracle import (  # noqa: F401
    partition_tiles,
    tile_origin,
    slice_tile,
    softmax_rows,
    attention_rows,
    attention,
    tile_attention,
    ramp_weight,
    blend,
    gate_score,
    cache_gate,
    similarity,
    StepState,
    denoise_step_tiled,
    rel_l1,
    accumulated_error,
    gain,
    GainState,
    gain_gate,
    gain_refresh,
    denoise_step_gain,
    tile_std,
    StdTracker,
    region_thresholds,
    shift_schedule,
    slice_tile_shifted,
    blend_shifted,
    fuse_and_denoise,
)
