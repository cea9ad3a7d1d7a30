"""MI355X-native hard-routed inference of Fast Feedforward (FFF) layers.

The work is done by hand-written HIP kernels behind a C ABI (include/fff.h,
built into libfff_hip.so).  This package is only the ctypes binding: it turns
torch tensors into device pointers and sizes.  There is no CPU fallback: if
the library cannot be loaded, importing the binding raises.
"""
from .binding import (ACT_GELU, ACT_RELU, DTYPE_BF16, DTYPE_F32, FffError, fff_bucket, fff_debug_option,
                      fff_descend, fff_forward_block, fff_forward_hard, fff_forward_hard_static, fff_forward_soft, fff_get_option, fff_last_launch,
                      fff_leaf_forward, fff_moe_top1_forward, fff_release_workspace, fff_reserve_workspace,
                      fff_reserve_workspace_bytes, fff_set_option, fff_set_workspace, fff_stage_times, fff_static_scratch_bytes,
                      fff_status_string, fff_version, fff_workspace_bytes, fff_workspace_bytes_moe,
                      fff_workspace_bytes_soft, lib, library_path)

__all__ = [
    "ACT_GELU", "ACT_RELU", "DTYPE_BF16", "DTYPE_F32", "FffError", "fff_bucket", "fff_debug_option", "fff_descend",
    "fff_forward_block", "fff_forward_hard", "fff_forward_hard_static", "fff_forward_soft", "fff_get_option", "fff_last_launch", "fff_leaf_forward",
    "fff_moe_top1_forward", "fff_release_workspace", "fff_reserve_workspace", "fff_reserve_workspace_bytes",
    "fff_set_option", "fff_set_workspace", "fff_stage_times", "fff_static_scratch_bytes", "fff_status_string", "fff_version",
    "fff_workspace_bytes", "fff_workspace_bytes_moe", "fff_workspace_bytes_soft", "lib", "library_path",
]
