"""MI355X-native diagonally-sparse linear layer (DynaDiag, arxiv 2506.11449): the forward product,
the two backward products and the TopK re-selection of diagonals, as hand-written HIP kernels for
gfx950 behind a C ABI (include/dynadiag.h).  This package is the Python binding of that ABI."""
from .binding import (DD_OP_BWD, DD_OP_BWD_INPUT, DD_OP_BWD_WEIGHT, DD_OP_BWD_WEIGHT_SCALED, DD_OP_DIAGHEUR, DD_OP_FWD, DD_OP_PREPARE,
                      DD_OP_SCALE_VALUES_BWD, DD_OP_SELECT, DD_ALGO_AUTO, DD_ALGO_BLOCKS, DD_ALGO_MATRIX, DD_ALGO_PREPARED, DD_ALGO_VECTOR, DD_BF16, DD_F32, DynaDiagError,
                      Prepared, PreparedShared, Workspace, dd_bwd_input, dd_bwd_input_shared, dd_bwd, dd_bwd_weight, dd_bwd_weight_scaled, dd_bwd_weight_static, dd_prepare_scaled, dd_select_soft, dd_static_scratch_bytes,
                      dd_diag_magnitude, dd_diagheur_update, dd_fwd, dd_fwd_shared, dd_prepare, dd_prepare_batched, dd_prepare_shared,
                      dd_scale_values, dd_scale_values_bwd, dd_select_diagonals, dd_select_prepare,
                      dd_soft_topk, dd_soft_topk_bwd, dd_workspace_bytes, load_library, make_layer)

__all__ = ["DD_OP_BWD", "DD_OP_BWD_INPUT", "DD_OP_BWD_WEIGHT", "DD_OP_BWD_WEIGHT_SCALED", "DD_OP_DIAGHEUR", "DD_OP_FWD", "DD_OP_PREPARE",
           "DD_OP_SCALE_VALUES_BWD", "DD_OP_SELECT", "DD_ALGO_AUTO", "DD_ALGO_BLOCKS", "DD_ALGO_MATRIX", "DD_ALGO_PREPARED", "DD_ALGO_VECTOR", "DD_BF16", "DD_F32", "DynaDiagError",
           "Prepared", "PreparedShared", "Workspace", "dd_bwd_input", "dd_bwd_input_shared", "dd_bwd", "dd_bwd_weight", "dd_bwd_weight_scaled", "dd_bwd_weight_static", "dd_prepare_scaled", "dd_select_soft", "dd_static_scratch_bytes",
           "dd_diag_magnitude", "dd_diagheur_update", "dd_fwd", "dd_fwd_shared", "dd_prepare", "dd_prepare_batched", "dd_prepare_shared",
           "dd_scale_values", "dd_scale_values_bwd", "dd_select_diagonals", "dd_select_prepare",
           "dd_soft_topk", "dd_soft_topk_bwd", "dd_workspace_bytes", "load_library", "make_layer"]
