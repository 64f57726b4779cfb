"""MI355X-native GAS layer step: hand-written HIP kernels behind a C ABI
(include/gas.h), with a ctypes binding of the same names."""
from .binding import (  # noqa: F401
    F32, BF16, GasError, Plan, HostTable, DiskTable, lib, gas_version,
    gas_pull, gas_push, gas_gcn_norm, gas_plan_create, gas_plan_destroy, gas_validate_indices,
    gas_spmm, gas_spmm_hist, gas_fuse_sources, gas_spmm_t,
    gas_linear, gas_mlp2, gas_linear_push, gas_mlp2_push, gas_mlp2_keep, gas_spmm_linear, spmm_linear_supported,
    gas_relu_bwd, gas_linear_bwd_input, gas_linear_bwd_weight, gas_linear_bwd_weight_workspace, gas_linear_bwd_weight_static,
    gas_softmax_xent, gas_sgd_step, gas_sq_norm, gas_sgd_step_clipped, gas_axpy, gas_row_distance, gas_row_distance_bwd, gas_row_dot,
    gas_pna_aggregate, gas_gat_aggregate, gas_pna_aggregate_bwd, gas_gat_aggregate_bwd)
