"""MI355X-native hot path of the Seer SpMV case study: six CSR SpMV schedules, one over the ELL and one over the COO
format (three of the eight with a preprocessing pass), the row-length feature reduction and the decision-tree
kernel selector, all inside libseer.so (hand-written HIP for gfx950) behind a C ABI;
this package is the thin Python binding over it."""
from .binding import (  # noqa: F401
    COO_WM, CSR_A, CSR_BM, CSR_S, CSR_MP, CSR_TM, CSR_WM, CSR_WO, ELL_TM, ONE_CALL_KERNELS, F_ITERATIONS, FEATURE_NAMES, NUM_DIRECT_KERNELS, NUM_FEATURES,
    NUM_KERNELS, DeviceCSR, Model, Plan, SeerError, Tree,
    alloc_workspace, ell_plan_bytes, slab_plan_bytes, features_workspace_bytes, kernel_name, lib, plan_bytes, seer_derive_features, seer_features,
    seer_known_features, seer_model_host_ns, seer_select, seer_tree_reachable, seer_spmv, seer_spmv_auto, seer_spmv_auto_result, seer_spmv_auto_static, STATIC_SCRATCH_BYTES, seer_spmv_model,
    seer_spmv_plan, seer_spmv_prepare, seer_spmv_prepared, seer_csr_check, seer_gather_sum, seer_stream_copy, seer_stream_sum, set_tuning,
    spmv_auto_workspace_bytes, spmv_prepared_workspace_bytes, spmv_workspace_bytes, strerror,
)
