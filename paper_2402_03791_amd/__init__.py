"""MI355X-native hot path of ZeroPP's pipeline + ZeRO-3 training: one pipeline stage run forward and
backward over a scheduling unit of micro-batches, flat-buffer gradient accumulation and a fused Adam
step, as hand-written gfx950 kernels behind a C ABI (include/zpp.h).  This package is the thin
Python binding (argument marshalling only); PyTorch supplies device memory and streams."""
from .binding import (Device, Stage, StageConfig, ZppError, lib, load_library, op_gemm_bf16_nt, op_gemm_bf16_tt, op_gemm_bf16_tt_group, op_gemm_bf16_nn, op_attention_fwd,
                      op_attention_bwd, op_attention_bwd_noalloc, op_flat_adam, op_flat_accumulate, op_flat_materialize, EXPORTS, profile_enable, profile_reset,
                      profile_read, PlanModel, plan_tp_comm, plan_zeropp_comm, plan_zeropp_wins, plan_bubbles, plan_max_memory,
                      plan_pp_method, plan_choose)

__all__ = ["Device", "Stage", "StageConfig", "ZppError", "lib", "load_library", "op_gemm_bf16_nt", "op_gemm_bf16_tt", "op_gemm_bf16_tt_group", "op_gemm_bf16_nn", "op_attention_fwd",
           "op_attention_bwd", "op_attention_bwd_noalloc", "op_flat_adam", "op_flat_accumulate", "op_flat_materialize", "EXPORTS", "profile_enable", "profile_reset", "profile_read",
           "PlanModel", "plan_tp_comm", "plan_zeropp_comm", "plan_zeropp_wins", "plan_bubbles", "plan_max_memory", "plan_pp_method",
           "plan_choose"]
