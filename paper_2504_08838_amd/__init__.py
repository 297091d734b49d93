"""MI355X-native hot path of a pruned draft model for speculative decoding.

Thin ctypes binding over ``libsd2.so`` (see ``include/sd2.h``); every step of the
path runs in the library's HIP kernels.  PyTorch is used by callers only to own
device memory and streams.
"""

from .binding import (  # noqa: F401
    SD2Error,
    BlobInfo,
    Matrix,
    ModelShape,
    Model,
    lib,
    lib_path,
    strerror,
    version,
    pack_sparse_size,
    pack_sparse,
    unpack_sparse,
    blob_info,
    blob_validate,
    matrix_init_sparse,
    matrix_init_dense,
    linear_workspace_size,
    sparse_linear,
    sparse_linear_partials,
    dense_linear,
    mlp_workspace_size,
    sparse_mlp_forward,
    model_create,
    model_destroy,
    drafter_workspace_size,
    sparse_drafter_forward,
    drafter_trace_size,
    sparse_drafter_forward_trace,
    drafter_forward_status,
    greedy_verify,
    check_token_ids_host,
    calibration_copy,
    lm_head_argmax,
    mask_gradient,
    prune_magnitude,
    draft_round,
    draft_round_status,
    draft_round_workspace_size,
    lm_head_workspace_size,
)
