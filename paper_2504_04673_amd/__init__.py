"""MI355X-native hot path of sparsity-aware block-row SpMM for full-graph GCN training.

The compute lives in libsagnn.so (hand-written HIP for gfx950, C ABI declared in
include/sagnn.h).  This package is a thin marshalling layer: torch supplies device memory
and the stream, every step runs in the library's kernels.  There is no CPU fallback: if the
library is missing or no GPU is present, calls raise.
"""
from .binding import (  # noqa: F401
    SagnnError, lib, lib_path, Plan, SpmmWorkspace, SpmmOptions, options_from_env, plan_buffers,
    spmm_plan_needed_rows, spmm_plan_needed_rows_noalloc, spmm_pack_rows, spmm_csr_prepare, spmm_csr_prepare_tuned, spmm_csr_tallskinny,
    dense_gemm_act, gcn_layer_fwd, gcn_layer_fwd_form, gcn_layer_bwd,
    ColBlocks, spmm_split_colblocks, spmm_stage_loop, spmm_volume_stats, spmm_csr_transpose,
    spmm_perm_from_labels, spmm_csr_permute_symmetric,
    ACT_IDENTITY, ACT_RELU, GEMM_FP32, GEMM_BF16, GEMM_FP32_BF16X3, PLAN_VALIDATE, PLAN_OBLIVIOUS, PLAN_MULTIPASS,
)
