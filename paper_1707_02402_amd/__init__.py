"""MI355X-native dynamic batching: program-tree execution engine and sparsely gated MoE layer.

Thin binding over libdynbatch.so (see include/dynbatch.h for the C ABI).
"""
from .binding import (DYNB_BF16, DYNB_F32, DYNB_PLAN_BALANCE, DYNB_PLAN_KEEP, DYNB_PLAN_PERSISTENT, DYNB_PLAN_THROUGHPUT, DYNB_SCHED_DEPTH, DYNB_SCHED_IMPROVED, DYNB_SCHED_NAIVE, DYNB_SCHED_STANDARD, DynbError,
                      Plan, dynbatch_backward, dynbatch_backward_workspace_bytes, dynbatch_classify, dynbatch_classify_workspace_bytes, dynbatch_execute, dynbatch_execute_check, dynb_set_spin_limit, dynbatch_pack_weights, dynbatch_packed_weights_bytes, dynbatch_plan, dynbatch_plan_dag, dynbatch_plan_device_bytes, dynbatch_plan_upload,
                      dynbatch_plan_view, dynbatch_workspace_bytes, dynb_timing_enable, dynb_timing_read, dynb_probe_copy, dynb_probe_mfma_bf16, dynb_probe_read,
                      moe_forward, moe_forward_static, moe_workspace_bytes, MOE_SEPARATE_PERMUTE, MOE_STAGES, MOE_STATIC_SCRATCH_BYTES)

__all__ = ["DYNB_BF16", "DYNB_F32", "DYNB_PLAN_BALANCE", "DYNB_PLAN_KEEP", "DYNB_PLAN_PERSISTENT", "DYNB_PLAN_THROUGHPUT", "DYNB_SCHED_DEPTH", "DYNB_SCHED_IMPROVED", "DYNB_SCHED_NAIVE", "DYNB_SCHED_STANDARD", "DynbError",
           "Plan", "dynbatch_backward", "dynbatch_backward_workspace_bytes", "dynbatch_classify", "dynbatch_classify_workspace_bytes", "dynbatch_execute", "dynbatch_execute_check", "dynb_set_spin_limit", "dynbatch_pack_weights", "dynbatch_packed_weights_bytes", "dynbatch_plan", "dynbatch_plan_dag", "dynbatch_plan_device_bytes", "dynbatch_plan_upload",
           "dynbatch_plan_view", "dynbatch_workspace_bytes", "dynb_timing_enable", "dynb_timing_read", "dynb_probe_copy", "dynb_probe_mfma_bf16", "dynb_probe_read", "moe_forward",
           "moe_forward_static", "moe_workspace_bytes", "MOE_SEPARATE_PERMUTE", "MOE_STAGES", "MOE_STATIC_SCRATCH_BYTES"]
