"""Fused array-combinator clusters on MI355X: HIP kernels behind a C ABI (include/fc.h) and its ctypes binding."""
from .binding import (FcError, Partition, fc_check, fc_cluster_kernel, fc_duplicate, fc_last_error, fc_num_edges,
                      fc_partition_check, fc_partition_trivial, fc_plan, fc_plan_greedy, fc_plan_weighted, fc_run_fused, fc_run_fused_static,
                      fc_run_unfused, fc_scratch_bytes, cost_vector)

__all__ = ["FcError", "Partition", "fc_check", "fc_cluster_kernel", "fc_duplicate", "fc_last_error", "fc_num_edges",
           "fc_partition_check", "fc_partition_trivial", "fc_plan", "fc_plan_greedy", "fc_plan_weighted", "fc_run_fused", "fc_run_fused_static",
           "fc_run_unfused", "fc_scratch_bytes", "cost_vector"]
