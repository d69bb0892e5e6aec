"""MI355X-native chunked sparse-attention decode path (LeoAM hot path).

The work is done by libleoam.so (hand-written HIP for gfx950, C ABI declared in
include/leoam.h).  `binding` exposes the entry points under the same names;
`DecodeLayer` is a small convenience holder of the per-layer buffers.
"""
from . import binding  # noqa: F401  (raises if the library is not built)
from .binding import (  # noqa: F401
    LeoamError, Shape, make_shape, kv_chunk_abstract_build, chunk_score, chunk_score_pin, chunk_topk_select,
    sparse_chunk_attention_decode, chunk_select_attention_decode, chunk_select_attention_decode_static,
    leoam_workspace_bytes,
    leoam_fused_workspace_bytes, leoam_fused_control_bytes, leoam_workspace_init, kv_chunk_abstract_append, leoam_tree_evaluations, chunk_tree_refine,
    leoam_tree_workspace_bytes, kv_chunk_compress, kv_chunk_recompress, chunk_compression_tags, leoam_compressed_bytes_bound, leoam_compression_share,
    leoam_validate_boundaries, leoam_copy_probe, leoam_read_probe,
    status_string, version, default_scale,
)
from .layer import DecodeLayer, DecodeStack  # noqa: F401
