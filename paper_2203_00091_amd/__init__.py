"""DFSS attention forward pass (arXiv 2203.00091) for AMD MI355X.

Thin Python binding over the C ABI of ``libdfss.so`` (see ``include/dfss.h``):
argument marshalling only, every step of the path runs in the HIP kernels.
PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    DFSS_BF16,
    DFSS_F32,
    DFSS_F32_BF16X3,
    DfssError,
    Shape,
    dense_attention,
    dense_attention_bias,
    dense_attention_fused,
    dense_attention_fused_bias,
    dense_attention_fused_blocked,
    dense_attention_fused_ragged,
    dense_workspace_bytes,
    dfss_attention,
    dfss_attention_backward,
    dfss_attention_bias,
    dfss_attention_blocked,
    dfss_attention_ragged,
    dfss_attention_staged,
    dfss_attention_staged_bias,
    dfss_attention_staged_static,
    dfss_static_scratch_bytes,
    dfss_backward_workspace_bytes,
    dfss_meta_bytes,
    dfss_meta_from_canonical,
    dfss_meta_to_canonical,
    dfss_sddmm_prune,
    dfss_sddmm_prune_bias,
    dfss_sparse_softmax,
    dfss_spmm,
    dfss_spmm_t,
    dfss_vals_bytes,
    dfss_workspace_bytes,
    library_path,
    load_library,
)
