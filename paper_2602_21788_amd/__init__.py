"""MI355X-native rank-local attention for Flexible Context Parallelism.

The product is libfcp.so (C ABI in include/fcp.h, HIP kernels under csrc/); `binding`
exposes the same entry points to Python and `rank` wires them into one rank's
forward / backward pass for tests and benchmarks.
"""
from .binding import (CostModel, FcpError, fcp_attn_bwd_delta, fcp_attn_bwd_step, fcp_attn_fwd_step,  # noqa: F401
                      fcp_grad_finalize, fcp_lse_merge, fcp_plan_groups, fcp_scratch_bytes, fcp_scratch_status,
                      fcp_shard_plan, fcp_shard_plan_mixed, fcp_mask_tables, fcp_attn_fwd_step_mixed,
                      fcp_attn_bwd_step_mixed, fcp_group_shard_args, fcp_attn_fwd_step_running,
                      fcp_attn_bwd_step_direct, fcp_grad_finalize_direct, fcp_attn_fwd_step_direct,
                      fcp_lse_merge_direct, fcp_attn_fwd_step_static)
