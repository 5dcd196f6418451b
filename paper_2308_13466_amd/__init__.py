"""MI355X-native SAT partition step: thin Python binding over libsat.so.

The library is the product; this package only marshals arguments. PyTorch is
used by callers for device memory and streams, never for the arithmetic.
"""
from .binding import (  # noqa: F401
    SatError, lib, lib_path, PartView, Predictor,
    partition_view_build, history_gather, history_gather_add, history_push, predict, predict_cached, predict_states, predict_states_workspace_bytes,
    predict_hop, predict_hop_workspace_bytes,
    predict_workspace_bytes, predictor_train_workspace_bytes, predictor_grad, sgd_update,
    history_compress_workspace_bytes, history_compress_plan, history_compress_encode,
    history_decompress, spmm_fwd, spmm_bwd, spmm_workspace_bytes,
    dense_fwd, dense_bwd, dense_bwd_workspace_bytes, loss_grad, gat_scores,
    gat_aggregate_fwd, gat_aggregate_bwd, gat_aggregate_bwd_workspace_bytes,
    loss_workspace_bytes, loss_grad_static, loss_grad_static_max_rows, status_string, version,
    F32, BF16, ACT_IDENTITY,
    ACT_RELU,
)
from .minibatch import minibatch_view  # noqa: F401
