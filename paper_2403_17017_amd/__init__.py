"""MI355X-native hot path of the Seer SpMV case study: four CSR SpMV schedules, the
row-length feature reduction and the decision-tree kernel selector, all inside
libseer.so (hand-written HIP for gfx950) behind a C ABI; this package is the thin
Python binding over it."""
from .binding import (  # noqa: F401
    CSR_BM, CSR_MP, CSR_TM, CSR_WM, CSR_WO, FEATURE_NAMES, NUM_FEATURES, NUM_KERNELS, DeviceCSR, Model, SeerError, Tree,
    alloc_workspace, features_workspace_bytes, kernel_name, lib, seer_derive_features, seer_features, seer_known_features,
    seer_select, seer_spmv, seer_spmv_model, seer_spmv_auto, seer_spmv_auto_result, spmv_auto_workspace_bytes, seer_stream_copy, seer_stream_sum, set_tuning, spmv_workspace_bytes, strerror,
)
