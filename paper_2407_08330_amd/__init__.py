"""Hierarchical document attention (HDT, arXiv 2407.08330) for AMD MI355X: hand-written HIP
kernels behind a C ABI (``include/hdt.h``), with a thin ctypes binding.  PyTorch is only used for
device memory and streams."""
from .binding import (  # noqa: F401
    HDT_EDGE_ALL,
    HDT_EDGE_DOWN,
    HDT_EDGE_SIBLING,
    HDT_EDGE_UP,
    HdtError,
    Layout,
    hdt_attn_bwd,
    hdt_attn_bwd_no_alloc,
    hdt_attn_bwd_workspace_bytes,
    hdt_attn_fwd,
    hdt_attn_fwd_workspace_bytes,
    hdt_build_cross_layout,
    hdt_build_layout,
    hdt_hpe_add,
    hdt_hpe_table,
    hdt_index_vectors,
    hdt_parents_from_levels,
    hdt_probe_mfma_bf16,
    hdt_release_cached_memory,
    hdt_timing_enable,
    hdt_timing_read,
    hdt_timing_reset,
    library_path,
    load_library,
)
