"""Python binding of libgcn_hip.so: same names as the C ABI in include/gcn.h, argument
marshalling only.  Tensors are torch CUDA(HIP) tensors used as device memory; every step of the
path runs inside the library's kernels on torch's current stream.

Importing this package does not load the library; the first call does, and raises if the
library has not been built (there is no CPU fallback).
"""
from .binding import (  # noqa: F401
    GcnError, Csr, lib, library_path, exported_symbols,
    gcn_csr_create, gcn_csr_create_from_csr, gcn_csr_create_from_csr_rect, gcn_spmm, gcn_spmm_static, gcn_spmm_pattern, gcn_scale_rows,
    gcn_csr_inv_sqrt_degrees, gcn_gemm, gcn_relu, gcn_relu_mask,
    gcn_softmax_nll, gcn_softmax_nll_masked, gcn_layer_forward, gcn_layer_backward, gcn_epoch, gcn_epoch_masked, gcn_epoch_preaggregated,
    gcn_epoch_workspace_bytes,
    gcn_epoch_view, gcn_config, gcn_csr_config, gcn_spmm_prepare, gcn_spmm_describe, gcn_epoch_prepare, gcn_scratch_release,
    gcn_build_count, gcn_csr_last_spmm_schedule, gcn_timing_read, gcn_timing_read_phases, gcn_version, gcn_last_spmm_schedule, gcn_radix_sort, gcn_exclusive_scan_i64, gcn_unique_u64,
    SCHED_ROWWISE, SCHED_SPLIT, SCHED_SWEEP, SCHED_HUB, SCHED_BLOCKED,
    SYMMETRISE, ADD_SELF_LOOPS, NORM_SYM, BUILD_TRANSPOSE, NORM_ROW,
    EPI_NONE, EPI_RELU, EPI_MASK, ORDER_AUTO, ORDER_GEMM_FIRST, ORDER_SPMM_FIRST, ACT_NONE, ACT_RELU,
    CFG_SPMM_ALGO, CFG_TIMING, CFG_SPMM_BLOCKS, CFG_SWEEP_HEAVY, CFG_SWEEP_WAVES, CFG_PATTERN_SPMM, CFG_HUB_MB, CFG_HUB_DMIN, CFG_HUB_BLOCK_COLS, CFG_SPLIT_LDS_KB, CFG_FUSED_LAST_LAYER,
)
