"""MI355X-native SampleAttention prefill hot path.

Thin Python binding over the C-ABI library ``libsampleattn.so`` (hand-written
HIP kernels for gfx950).  The binding only marshals arguments: every step of
the path runs in the library's kernels.  PyTorch supplies device memory and the
stream, nothing else.
"""
from .binding import (  # noqa: F401
    SA_OUT_BF16,
    SA_OUT_F32,
    SA_KERNELS,
    SaError,
    SampleAttentionPlan,
    Shape,
    lib_path,
    block_sample_attention,
    chunked_sample_attention,
    load_library,
    n_blocks,
    sa_block_scores,
    sa_block_sparse_attn,
    sa_select_blocks,
    sa_select_chunked,
    sa_sparse_attn_chunked,
    sa_dense_attn,
    sa_dense_attn_static,
    SA_STATIC_SCRATCH_BYTES,
    sa_probe_copy,
    sa_probe_mfma,
    sa_profile_enable,
    sa_profile_read,
    sa_rows_from_ratio,
    sa_sample_scores,
    sa_select_strips,
    sa_sparse_attn,
    sa_sparse_attn_partitioned,
    sa_partitioned_workspace_bytes,
    sa_workspace_bytes,
    sample_attention,
)
