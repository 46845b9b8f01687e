"""N:M-sparse linear layer for AMD MI355X: thin Python binding over the C ABI in include/nm_sparse.h.

Importing the package does not load the HIP library; the first call does, and fails loudly if the
library has not been built (python -m paper_2409_09708_amd.build).
"""
from .binding import (  # noqa: F401
    NmError,
    bf16_bits,
    bf16_tensor,
    library_path,
    load_library,
    nm_config_cost,
    nm_index_bytes,
    nm_backward_weight_workspace_bytes,
    nm_linear_backward_input,
    nm_linear_backward_weight,
    nm_linear_forward,
    nm_linear_forward_prepared,
    nm_spmm_prepare,
    nm_mask_bytes,
    nm_mask_check,
    nm_pack,
    nm_pack_batched,
    nm_pack_prepare_batched,
    nm_pack_ranked,
    nm_prune,
    nm_rank,
    nm_sample_config,
    nm_rank_batched,
    nm_rank_bytes,
    nm_rank_mask,
    nm_spmm,
    nm_spmm_workspace_bytes,
    nm_status_string,
    nm_unpack,
    nm_values_bytes,
)
