"""CPU oracle for the SBP hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this.  Only tests, the smoke check
and the benchmark's cpu_baseline leg call it.  It shares no code with the HIP
path; it is a plain fp64 write-out of what the paper defines.
"""
from .sbp_oracle import (  # noqa: F401
    GRID_PER_CELL,
    GRID_SHARED,
    RANDOM_MASK,
    TEMPORAL,
    random_keep_count,
    sample_indices_random,
    temporal_keep_frames,
    sample_indices_temporal,
    k_from_ratio,
    keep_count,
    sample_indices,
    sample_indices_cells,
    keep_count_cells,
    inverse_map,
    forward_cache,
    backward_linear,
    backward_dwconv,
    mix64,
    gelu,
    gelu_grad,
    act_forward_rows,
    act_backward_rows,
    layernorm_rows,
    backward_layernorm,
    backward_layerscale,
    forward_cache_patches,
    attention_scores,
    backward_attention,
    backward_downsample,
)
