"""MI355X-native hot path of discrete-time dynamic-GNN training: on-GPU snapshot reconstruction
from a graph difference, the GCN step A~ (X W), and TM-GCN's M-transform.

Everything is computed by hand-written HIP kernels behind the C boundary declared in
include/dgnn.h; this package only marshals torch tensors (used for device memory and streams)
into those calls.  There is no CPU fallback: without the built library the calls raise.
"""
from .binding import (  # noqa: F401
    DgnnError, build_library, library_path, load_library, strerror,
    # the hot path
    csr_validate, csr_dinv, delta_h2d, delta_rebuild, delta_rebuild_workspace, feature_transform, spmm, spmm_workspace, spmm_static,
    spmm_static_limit, mproduct,
    # its backward half, and a series processed in blocks
    mproduct_backward, mproduct_block, mproduct_backward_block, relu_backward, weight_grad, weight_grad_workspace,
    input_grad, csr_transpose, coo_transpose,
    # snapshots that carry values; smoothing on the device
    delta_rebuild_weighted, spmm_weighted, csr_weighted_dinv, csr_weighted_dinv_workspace, csr_combine,
    csr_combine_workspace,
    # CD-GCN layer and the LSTM over weights
    concat_relu, transform_concat_relu, transform_concat_relu_supported, lstm_cell, lstm_step, lstm_step_supported, lstm_cell_backward, lstm_step_backward,
    lstm_step_backward_supported, concat_relu_backward, bias_grad, bias_grad_workspace, add,
    DGNN_VALIDATE, DGNN_UPDATES_SORTED, DGNN_RELU, DGNN_H_PRESCALED, DGNN_F32, DGNN_BF16,
)
