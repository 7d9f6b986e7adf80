"""MI355X (gfx950) bf16 GEMM + fused-epilogue library: Python binding of the C ABI.

Every computation runs in the HIP kernels of libfact_gemm.so; this package only marshals
arguments.  There is no CPU or PyTorch fallback: if the library is not built, loading fails.
"""
from .binding import (  # noqa: F401
    ACT_GELU_TANH, ACT_NONE, ACT_SILU_GATE, FactError, Epilogue, lib, lib_path,
    fact_gemm, fact_gemm_batched, fact_gemm_splitk, fact_gemm_splitk_workspace_bytes, fact_gemm_f32out_workspace_bytes,
    fact_block_mlp, fact_block_mlp_f16, fact_block_mlp_workspace_bytes, fact_gemm_ex, fact_attention,
    fact_norm, fact_rope, Block, fact_block_scratch_bytes, fact_block_scratch_offsets, fact_block_forward,
    fact_num_configs, fact_config_info, fact_select_config,
    fact_gemm_splitk_static, fact_gemm_splitk_static_init, fact_gemm_splitk_static_capacity, fact_tail_timeouts, fact_test_tail_poll_budget, fact_tune_persistent, fact_persistent_grid, fact_registry_load, fact_registry_clear, fact_registry_size, CONFIG_TABLE, CONFIG_GUARDED,
    fact_status_string, fact_last_error, fact_version,
)
