"""PCSR SpMM for AMD MI355X: Python face of the C-ABI library libpcsr.so.

The library is loaded on first use and there is no fallback: a missing or unloadable
libpcsr.so raises.
"""
from .binding import (FEATURE_NAMES, PCSR_FLAG_ATOMIC_SPLIT, PCSR_FLAG_COLUMN_ORDER, PCSR_FLAG_DEVICE_CSR, PCSR_FLAG_GPU_BUILD, PCSR_FLAG_HOST_ONLY,  # noqa: F401
                      PCSR_FLAG_NO_VALIDATE, PCSR_FLAG_NO_XCD_REMAP, PCSR_FLAG_WINDOW_IF_USEFUL, Handle, PcsrError, make_params,
                      pcsr_build, pcsr_export, pcsr_export_schedule, pcsr_features, pcsr_free, pcsr_mac_job_gap,
                      pcsr_params_t, pcsr_permute_csr, pcsr_query_launch, pcsr_reorder, pcsr_reorder_by_degree, pcsr_select, pcsr_set_kernel_params,
                      pcsr_reserve_workspace, pcsr_spmm, pcsr_spmm_static, pcsr_static_scratch_bytes, pcsr_strerror, pcsr_transpose_csr, pcsr_window_stats,
                      pcsr_workspace_bytes)
