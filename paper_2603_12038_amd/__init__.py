"""MI355X-native decode-attention hot path of Slow-Fast Inference (libsfi + a thin ctypes binding)."""
from .binding import (SfiConfig, SfiContext, SfiError, load_library, sfi_advance, sfi_create, sfi_dense_attn, sfi_dense_attn_floor,  # noqa: F401
                      sfi_destroy, sfi_device_status, sfi_evidence_add, sfi_evidence_add_causal, sfi_evidence_select, sfi_fast_step, sfi_fast_step_compact, sfi_fast_step_floor, sfi_fast_step_static, sfi_mixed_step, sfi_mixed_step_compact, sfi_mixed_step_desc, sfi_step_begin, sfi_plan_splits, sfi_query_splits, sfi_reorg, sfi_set_block_table, sfi_set_profiling,
                      sfi_set_dense_k_layout, sfi_set_tuning, sfi_slow_attn, sfi_slow_select, sfi_slow_step, sfi_stage_times, sfi_strerror, sfi_trigger, sfi_workspace_bytes)
