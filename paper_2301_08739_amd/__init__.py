"""MI355X-native Flattened Window Attention: thin Python binding over libflatformer.so.

Every step of the path (key generation, radix argsort, grouping, gather, the attention layer,
scatter) runs in the library's HIP kernels; this package only marshals arguments.  PyTorch is
used for device memory and streams.  There is no CPU fallback: calling anything here without the
built library raises.
"""
from .binding import (Geometry, Geometry3, VoxelGrid, LayerWeights, FF_F32, FF_BF16, FF_F16, FF_FLAG_OUT_F32, FF_FLAG_FORCE_GENERIC,
                      FF_FLAG_TAIL_DROP, FF_TAIL_MASK, FF_TAIL_DROP,
                      FF_FLAG_VARIANT,
                      FlatformerError, load_library, library_path, exported_symbols,
                      ff_flatten, ff_check_coords, ff_flatten_batch, ff_flatten_batch_workspace_bytes, ff_group_attention_path,
                      FF_PATH_PLAIN, FF_PATH_FUSED, ff_flatten_noalloc, FF_NOALLOC_SCRATCH_BYTES, ff_flatten3d, ff_flatten_workspace_bytes, ff_group_attention,
                      ff_group_attention_workspace_bytes, ff_gather, ff_scatter, ff_bev_scatter, ff_voxelize,
                      ff_voxelize_workspace_bytes, ff_fwa_block,
                      ff_fwa_block_workspace_bytes, ff_status_string, ff_version)

__all__ = [
    "Geometry", "Geometry3", "VoxelGrid", "LayerWeights", "FF_F32", "FF_BF16", "FF_F16", "FF_FLAG_OUT_F32", "FF_FLAG_FORCE_GENERIC", "FF_FLAG_VARIANT",
    "FF_FLAG_TAIL_DROP", "FF_TAIL_MASK", "FF_TAIL_DROP",
    "FlatformerError", "load_library", "library_path", "exported_symbols",
    "ff_flatten", "ff_check_coords", "ff_flatten_batch", "ff_flatten_batch_workspace_bytes", "ff_group_attention_path",
    "FF_PATH_PLAIN", "FF_PATH_FUSED", "ff_flatten_noalloc", "FF_NOALLOC_SCRATCH_BYTES", "ff_flatten3d", "ff_flatten_workspace_bytes", "ff_group_attention",
    "ff_group_attention_workspace_bytes", "ff_gather", "ff_scatter", "ff_bev_scatter", "ff_voxelize", "ff_voxelize_workspace_bytes", "ff_fwa_block",
    "ff_fwa_block_workspace_bytes", "ff_status_string", "ff_version",
]
