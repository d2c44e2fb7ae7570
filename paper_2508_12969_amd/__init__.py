"""Compact Attention block-sparse forward for MI355X: HIP kernels behind a C ABI.

The product is `libcompact_attn.so` (sources under `csrc/`, interface in
`include/compact_attn.h`); this package only builds it and marshals arguments.
"""
from .binding import (  # noqa: F401
    CompactAttnError,
    Layout,
    compact_attn_build_layout,
    compact_attn_dense,
    compact_attn_forward,
    compact_attn_forward_natural,
    compact_attn_forward_static,
    compact_attn_free_layout,
    compact_attn_last_error,
    compact_attn_layout_csr,
    compact_attn_layout_from_csr,
    compact_attn_layout_info,
    compact_attn_layout_order,
    compact_attn_layout_pairs,
    compact_attn_layout_packing,
    compact_attn_layout_similarity,
    compact_attn_layout_union,
    compact_attn_layout_upload,
    compact_attn_permute,
    compact_attn_search_head,
    compact_attn_tile_mass,
    library_path,
    load_library,
)
