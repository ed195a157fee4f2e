"""MI355X-native DPSGD gradient privatisation: thin ctypes binding over libdp_privatise.so.

Every function here only marshals arguments (device pointers of torch tensors, sizes, the
current HIP stream) into the C ABI declared in include/dp_privatise.h; all arithmetic runs
in the library's HIP kernels.  There is no CPU fallback: if the library has not been built
or cannot be loaded, importing the binding's functions raises.
"""
from .binding import (DP_BF16, DP_CONV2D, DP_DENSE, DP_F32, DP_GN_AFFINE, DP_NCHW, DP_NHWC,
                      DP_WS_PER_EXAMPLE_GRAD, DP_WS_RECOMPUTE, DP_VARIANT_SHARED, DP_VARIANT_MATERIALISE, DpError, LayerDesc, dp_add_noise_finalize,
                      dp_bias_count, dp_group_clip_bounds, dp_clip_accumulate, dp_clip_accumulate_recompute, dp_clip_factors,
                      dp_add_noise_finalize_update, dp_add_noise_finalize_flat, TensorTable, dp_add_example_noise, dp_clip_accumulate_segments, SegmentTable, dp_kernel_variant, dp_last_error, dp_norms, dp_norm_partial_count, dp_norms_from_partials, dp_layer_norms_from_partials, dp_unit_grad, dp_unit_grad_batch, dp_unit_workspace_bytes,
                      dp_per_example_grad_partials, dp_per_example_grad_batch, dp_clip_accumulate_recompute_batch, LayerBatch, PartialTable, dp_per_example_grad, dp_per_example_grad_static, dp_static_scratch_bytes, dp_philox_raw, dp_profile_next_contraction, dp_version,
                      dp_weight_count, dp_workspace_bytes, lib_path, load_library, make_desc)
from .pipeline import PrivatiseStep

__all__ = [
    "DP_BF16", "DP_CONV2D", "DP_DENSE", "DP_F32", "DP_GN_AFFINE", "DP_NCHW", "DP_NHWC",
    "DP_WS_PER_EXAMPLE_GRAD", "DP_WS_RECOMPUTE", "DP_VARIANT_SHARED", "DP_VARIANT_MATERIALISE", "DpError", "LayerDesc", "dp_add_noise_finalize",
    "dp_bias_count", "dp_group_clip_bounds", "dp_clip_accumulate", "dp_clip_accumulate_recompute", "dp_clip_factors",
    "dp_add_noise_finalize_update", "dp_add_noise_finalize_flat", "TensorTable", "dp_add_example_noise", "dp_clip_accumulate_segments", "SegmentTable", "dp_kernel_variant", "dp_last_error", "dp_norms", "dp_norm_partial_count", "dp_norms_from_partials", "dp_layer_norms_from_partials", "dp_unit_grad", "dp_unit_grad_batch", "dp_unit_workspace_bytes",
    "dp_per_example_grad_partials", "dp_per_example_grad_batch", "dp_clip_accumulate_recompute_batch", "LayerBatch", "PartialTable", "dp_per_example_grad", "dp_per_example_grad_static", "dp_static_scratch_bytes", "dp_philox_raw", "dp_profile_next_contraction", "dp_version", "dp_weight_count",
    "dp_workspace_bytes", "lib_path", "load_library", "make_desc", "PrivatiseStep",
]
