"""Thin Python binding of libhspmd_attn (argument marshalling only).

Every step of the hot path runs inside the HIP library; PyTorch appears here only as the owner
of device memory and streams.  There is no CPU fallback: if the shared library is missing or no
GPU is present, the compute calls raise.
"""
from .binding import (  # noqa: F401
    HspmdError, Plan, LIST_FWD, LIST_DQ, LIST_DKV, GRAD_BF16, GRAD_F32, ORDER_XCD_COST, ORDER_NATURAL, ORDER_COST,
    library_path, load_library, build_cu_seqlens, schedule, tile_rows,
    attn_varlen_fwd, attn_varlen_bwd, profile_enable, profile_read, profile_read_stats, probe_scratch_bytes, probe_mfma_tflops,
    BlockPlan, block_schedule, attn_block_fwd, attn_merge, attn_block_bwd, estimate_ms,
    rope_table_bytes, rope_table, rope_qk, attn_varlen_bwd_rope, attn_block_bwd_rope,
    attn_varlen_bwd_static_ws, STATIC_WORKSPACE_BYTES, probe_mfma_rate, PROBE_MODES,
)
