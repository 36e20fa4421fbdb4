"""KNN-softmax output layer for extreme classification on one MI355X: thin Python binding over the
C-ABI library `libknnsoftmax.so` (hand-written HIP for gfx950).  See include/knnsoftmax.h for the contract
of every call; this package only marshals arguments (torch tensors provide device memory and streams)."""
from . import binding  # noqa: F401
from .binding import (KS_DEV_RANGE, FLAG_UNIT_ROWS, FLAG_PAD_RANDOM, FLAG_TRUSTED_LIST, knn_graph_compress, knn_select_active_csr, knn_graph_update,
                      knn_graph_update_workspace, knn_softmax_bwd_from_stats, knn_softmax_fwd_stats, knn_softmax_fwd_bwd_update,
                      knn_softmax_fwd_bwd_update_selected, knn_softmax_selected_workspace,
                      knn_softmax_fwd_bwd_update_selected_next, knn_softmax_selected_next_workspace,
                      knn_softmax_bwd_from_stats_next, knn_softmax_split_next_workspace,
                      knn_softmax_split_workspace,
                      knn_select_active_csr_workspace, KS_DEV_BAD_COUNT, KS_DEV_BAD_GRAPH_ID, KS_DEV_BAD_INDEX, KS_DEV_BAD_LABEL,  # noqa: F401
                      KS_DEV_IDX_NOT_SORTED, KS_INVALID_ARG, KS_OK, KS_UNSUPPORTED, KS_WORKSPACE_TOO_SMALL,
                      KsError, apply_weight_grad, apply_weight_grad_normalized, apply_weight_grad_normalized_workspace,
                      apply_weight_grad_workspace, knn_norm_backward_rows, knn_normalize_rows, full_softmax_fwd_bwd,
                      full_softmax_workspace, knn_gather_rows, knn_graph_build, knn_graph_build_plan, knn_graph_build_workspace,
                      knn_select_active, knn_select_active_static, knn_select_workspace, knn_softmax_fwd_bwd, knn_softmax_workspace,
                      ks_version, lib, lib_path, GradTopkPlan, grad_topk_plan, grad_topk_select)
