"""Fused attention for AMD MI355X (gfx950): thin Python binding over the C-ABI library.

The HIP library (libflat_attn.so, built in-tree by `paper_2107_06419_amd.build`) does all the
work; this package only marshals arguments.  There is no CPU or PyTorch fallback: if the
library is missing, every call raises.
"""
from .binding import (FLAT_MASK_CAUSAL, FLAT_MASK_NONE, FlatAttnError, flat_attn_fwd, flat_attn_fwd_cross, flat_attn_fwd_blocksparse, flat_attn_fwd_f32,
                      flat_attn_status_string, flat_attn_unfused, flat_attn_unfused_workspace_bytes,
                      flat_attn_version, library_path, load_library, probe_library_path, load_probe_library, flat_attn_mfma_probe, flat_attn_mfma_probe_flops,
                      flat_attn_mfma_probe_sink_bytes, FlatTileShape, flat_attn_tile_shape_count,
                      flat_attn_tile_shape_get, flat_attn_tile_shape_occupancy, flat_attn_tile_shape_default, flat_attn_fwd_tile, flat_attn_mix_probe,
                      flat_attn_mix_probe_flops, flat_attn_mix_probe_sink_bytes, flat_attn_mix_probe_src_bytes,
                      flat_attn_fwd_splitkv, flat_attn_fwd_splitkv_splits, flat_attn_fwd_splitkv_workspace_bytes,
                      flat_attn_fwd_splitkv_static, FLAT_SPLITKV_STATIC_BYTES)

__all__ = ["FLAT_MASK_NONE", "FLAT_MASK_CAUSAL", "FlatAttnError", "flat_attn_fwd", "flat_attn_fwd_cross", "flat_attn_fwd_blocksparse", "flat_attn_fwd_f32",
           "flat_attn_unfused", "flat_attn_unfused_workspace_bytes", "flat_attn_status_string", "flat_attn_version",
           "library_path", "load_library", "probe_library_path", "load_probe_library", "flat_attn_mfma_probe", "flat_attn_mfma_probe_flops",
           "flat_attn_mfma_probe_sink_bytes", "FlatTileShape", "flat_attn_tile_shape_count", "flat_attn_tile_shape_get",
           "flat_attn_tile_shape_occupancy", "flat_attn_tile_shape_default", "flat_attn_fwd_tile", "flat_attn_mix_probe", "flat_attn_mix_probe_flops",
           "flat_attn_mix_probe_sink_bytes", "flat_attn_mix_probe_src_bytes", "flat_attn_fwd_splitkv",
           "flat_attn_fwd_splitkv_splits", "flat_attn_fwd_splitkv_workspace_bytes", "flat_attn_fwd_splitkv_static",
           "FLAT_SPLITKV_STATIC_BYTES"]
