"""MI355X-native H-SADMM structured-sparsity step: thin Python binding over libhsadmm.so.

Every step of the path runs in the HIP kernels of csrc/hsadmm.hip; this package only marshals
arguments (see include/hsadmm.h for the contract).  There is no CPU fallback: loading fails loudly when
the library has not been built.
"""
from .binding import (  # noqa: F401
    HsadmmError, Plan, LIB_PATH, load_library, build_library, exported_symbols,
    hsadmm_project, hsadmm_project_compact, hsadmm_compact, hsadmm_expand, hsadmm_strerror, hsadmm_version,
    hsadmm_kernel_timing_enable, hsadmm_kernel_timing_read, hsadmm_kernel_grids, hsadmm_plan_estimates, hsadmm_project_frozen, hsadmm_project_frozen_compact, hsadmm_mask_or, hsadmm_compact_sum, hsadmm_node_coefficients,
    hsadmm_plan_set_node_weights, hsadmm_project_weighted, hsadmm_project_weighted_compact, hsadmm_project_weighted_frozen, hsadmm_project_weighted_frozen_compact, hsadmm_dual_inter, hsadmm_residuals, hsadmm_average, hsadmm_mask_drift, hsadmm_expand_dual, hsadmm_retrain_project, hsadmm_retrain_expand, hsadmm_adapt_penalties, hsadmm_scale_layers,
    hsadmm_project_compact_static, hsadmm_step, hsadmm_selection_from_mask, hsadmm_layer_sqnorms, hsadmm_stopping_test,
    MODE_NONE, MODE_FILTER, MODE_CHANNEL, MODE_BOTH, MAX_REPLICAS,
)
