"""Thin Python binding of libprism (fused RMSNorm -> MatMul family for MI355X).

Argument marshalling only: every step of the computation runs in the HIP
kernels behind the C ABI declared in ``include/prism.h``.  There is no CPU or
PyTorch fallback; if the shared library is missing the import fails.
"""
from .binding import (  # noqa: F401
    PRISM_BF16,
    PRISM_F32,
    PRISM_F16,
    PRISM_OP_RMSNORM_GATED_MLP,
    PRISM_OP_RMSNORM_MATMUL,
    PRISM_OP_SOFTMAX_MATMUL,
    PRISM_PATH_AUTO,
    PRISM_PATH_DECODE,
    PRISM_PATH_PREFILL,
    PRISM_PATH_ROWS,
    PRISM_PATH_ATTENTION,
    PRISM_PATH_SIMPLE,
    PrismError,
    Plan,
    ensure_workspace,
    lib,
    library_path,
    prism_plan,
    prism_plan_table_clear,
    prism_plan_table_set,
    prism_plan_table_size,
    prism_rmsnorm_gated_mlp,
    prism_rmsnorm_glu,
    prism_swiglu,
    prism_softmax_matmul,
    prism_gqa_decode_attention,
    prism_attention_plan,
    prism_rmsnorm_matmul,
    prism_set_override,
    prism_set_stream_balance,
    prism_stream_partition_blocks,
    prism_set_workspace,
    prism_status_string,
    prism_version,
    prism_workspace_bytes,
)
