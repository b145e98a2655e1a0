"""MI355X-native HALO group-sparse FFN path: thin Python binding over libhalo.so.

The functions here have the names of the C entry points (see include/halo.h) and do
argument marshalling only; every step of the path runs in the HIP kernels.  PyTorch
tensors are used for device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    HaloError, Shape, MhaShape, halo_mha_workspace_bytes, halo_head_sparse_mha, halo_mha_forward, halo_mha_forward_ahead, halo_build_schedule, halo_workspace_bytes, halo_workspace_bytes_q4, halo_predict_scores,
    halo_build_group_mask, halo_group_sparse_ffn, halo_ffn_forward, halo_ffn_forward_ahead,
    halo_ffn_forward_static, halo_static_scratch_bytes,
    halo_group_sparse_ffn_q4, halo_ffn_forward_q4, halo_ffn_forward_ahead_q4,
    halo_profile_begin, halo_peak_read_stream, halo_peak_mfma_bf16, halo_stack_residual_norm,
    halo_profile_end, halo_ratios_comp_greedy, halo_ratios_min_max, library_path, load_library, pack_down_proj, prepared,
)
