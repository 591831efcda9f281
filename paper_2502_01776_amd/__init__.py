"""MI355X-native sparse 3D attention (Sparse VideoGen hot path).

The package is a thin ctypes binding over the C-ABI library built from csrc/.
Nothing is loaded at import time; `binding.lib()` loads the shared object on first
use and raises if it has not been built.
"""
from .binding import (SvgShape, SVG_HEAD_SPATIAL, SVG_HEAD_TEMPORAL, SVG_LIST_TEMPORAL_FRAME_MAJOR, SVG_ATTN_QO_TOKEN_ORDER, SVG_ATTN_ELEMENT_MASK, SVG_ATTN_KV_TOKEN_ORDER, SvgError, lib, shape_from_config,
                      svg_tile_list_build, svg_tile_counts, svg_workspace_bytes, svg_profile_plan, svg_profile_heads, svg_profile_heads_static, SVG_STATIC_SCRATCH_BYTES,
                      svg_layout_fwd, svg_layout_inv, svg_sparse_attn_fwd, svg_sparse_attn_fwd_ex, svg_dense_attn_fwd, svg_fp8_buffer_bytes, svg_fp8_quantize,
                      svg_sparse_attn_fp8_fwd, svg_qk_norm_rope, SVG_NORM_NONE, SVG_NORM_RMS, SVG_NORM_LAYER,
                      SVG_ROPE_INTERLEAVED, SVG_ROPE_HALF, SVG_FP8_Q, SVG_FP8_K, SVG_FP8_VT, SVG_FP8_SCALES,
                      svg_strerror, svg_version, svg_probe_mfma_bf16, svg_probe_lds, svg_layout_kv_temporal, svg_sparse_attn_fwd_kv2)

__all__ = ["SvgShape", "SVG_HEAD_SPATIAL", "SVG_HEAD_TEMPORAL", "SVG_LIST_TEMPORAL_FRAME_MAJOR", "SVG_ATTN_QO_TOKEN_ORDER", "SVG_ATTN_ELEMENT_MASK", "SVG_ATTN_KV_TOKEN_ORDER", "SvgError", "lib", "shape_from_config",
           "svg_tile_list_build", "svg_tile_counts", "svg_workspace_bytes", "svg_profile_plan", "svg_profile_heads", "svg_profile_heads_static", "SVG_STATIC_SCRATCH_BYTES",
           "svg_layout_fwd", "svg_layout_inv", "svg_sparse_attn_fwd", "svg_sparse_attn_fwd_ex", "svg_dense_attn_fwd", "svg_fp8_buffer_bytes", "svg_fp8_quantize",
           "svg_sparse_attn_fp8_fwd", "svg_qk_norm_rope", "SVG_NORM_NONE", "SVG_NORM_RMS", "SVG_NORM_LAYER",
           "SVG_ROPE_INTERLEAVED", "SVG_ROPE_HALF", "SVG_FP8_Q", "SVG_FP8_K", "SVG_FP8_VT", "SVG_FP8_SCALES",
           "svg_strerror", "svg_version", "svg_probe_mfma_bf16", "svg_probe_lds", "svg_layout_kv_temporal", "svg_sparse_attn_fwd_kv2"]
