"""MI355X-native library for the server-side hot path of MLfabric
(arXiv 1907.00434): ordered K-way aggregate, ordered server apply, fused
aggregate + apply and the LDA count-delta scatter-add.

The work is done by hand-written HIP kernels behind a C ABI
(``include/mlfabric.h``); this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    MLF_MAX_K,
    MlfError,
    library_path,
    mlf_aggregate,
    mlf_aggregate_apply,
    mlf_aggregate_norm,
    mlf_aggregate_update_norms,
    mlf_apply_grouped,
    mlf_apply_grouped_norms,
    mlf_apply_grouped_update_norms,
    mlf_counts_add_dense,
    mlf_divergence,
    mlf_divergence_bound,
    mlf_divergence_static,
    mlf_norms_workspace_bytes,
    mlf_update_norms_workspace_bytes,
    mlf_apply_ordered,
    mlf_sparse_scatter_add,
    mlf_sparse_workspace_bytes,
    mlf_status_string,
    raw,
)
