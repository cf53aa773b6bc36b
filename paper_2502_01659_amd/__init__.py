"""sga: sparse graph attention for AMD MI355X (gfx950).

Thin Python binding over the C ABI of libsga.so (include/sga.h).  Every step of
the attention path runs in the HIP kernels; Python only marshals arguments, and
PyTorch only provides device memory and streams.
"""
from .binding import (SgaError, PATH_AUTO, PATH_GATHER, PATH_TILE, PATH_TILE_SPLIT, load, lib_path,
                      mask_nnz, build_mask, validate_csr, workspace_bytes, alloc_workspace,
                      attention_forward, attention_forward_implicit,
                      attention_accumulate, attention_accumulate_implicit,
                      sga_attention_accumulate, sga_attention_accumulate_implicit,
                      sga_mask_nnz, sga_build_mask, sga_validate_csr, sga_workspace_bytes,
                      sga_attention_forward, sga_attention_forward_implicit,
                      sga_status_string, sga_profile_enable, sga_profile_collect, sga_profile_last_kernel,
                      GraphPlan, GRAPH_TILES_COVER_ALL, GRAPH_TILE_PARTS_FIT, GRAPH_ROW_CHUNKS_FIT,
                      graph_prepare, attention_forward_prepared, attention_accumulate_prepared,
                      sga_graph_prepare, sga_attention_forward_prepared,
                      sga_attention_accumulate_prepared,
                      sga_static_scratch_init, sga_static_scratch_bytes, sga_attention_forward_static)

__all__ = [
    "SgaError", "PATH_AUTO", "PATH_GATHER", "PATH_TILE", "PATH_TILE_SPLIT", "load", "lib_path",
    "mask_nnz", "build_mask", "validate_csr", "workspace_bytes", "alloc_workspace",
    "attention_forward", "attention_forward_implicit",
    "attention_accumulate", "attention_accumulate_implicit",
    "sga_attention_accumulate", "sga_attention_accumulate_implicit",
    "sga_mask_nnz", "sga_build_mask", "sga_validate_csr", "sga_workspace_bytes",
    "sga_attention_forward", "sga_attention_forward_implicit", "sga_status_string",
    "sga_profile_enable", "sga_profile_collect", "sga_profile_last_kernel",
    "GraphPlan", "GRAPH_TILES_COVER_ALL", "GRAPH_TILE_PARTS_FIT", "GRAPH_ROW_CHUNKS_FIT",
    "graph_prepare", "attention_forward_prepared", "attention_accumulate_prepared",
    "sga_graph_prepare", "sga_attention_forward_prepared", "sga_attention_accumulate_prepared",
    "sga_static_scratch_init", "sga_static_scratch_bytes", "sga_attention_forward_static",
]
