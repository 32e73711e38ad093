"""MI355X-native one-GPU MoE-layer forward (libmoe) and its thin Python binding.

The HIP kernels live in csrc/ behind the C-ABI declared in include/moe.h and
include/moe_sched.h, include/moe_train.h, include/moe_offload.h, include/moe_comm.h; this
package only marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (ACT, DTYPE, MoeError, Shape, alloc_buffers, lib, lib_path,
                      moe_calib_copy, moe_calib_gemm, moe_calib_mfma, moe_capacity, moe_expert_gemm_kernel, moe_combine, moe_dispatch, moe_dispatch_static,
                      moe_dispatch_static_limit, moe_expert_ffn,
                      moe_last_error, moe_layer_chunked, moe_max_rows, moe_pack_gate,
                      moe_pack_weights, moe_packed_gate_bytes, moe_packed_weight_bytes,
                      moe_profile_enable, moe_profile_read, moe_route, moe_tune_ffn_group_rows,
                      moe_workspace_bytes,
                      STAGES)

from .sched_binding import (PathShape, moe_devices_for_expert, moe_path_count, moe_path_finalize,
                            moe_path_profile, moe_popularity_estimate, moe_schedule_experts,
                            moe_schedule_layer, moe_top_lists_identical)

from .offload_binding import (moe_expert_ffn_offloaded, moe_offload_staging_bytes,
                              moe_offload_workspace_bytes)
from .train_binding import (moe_backward_workspace_bytes, moe_layer_backward,
                            moe_layer_forward_keep)
from . import comm_binding as comm
from .comm_binding import moe_layer_padded, moe_padded_workspace_bytes

__all__ = ["comm", "moe_layer_padded", "moe_padded_workspace_bytes", "moe_expert_ffn_offloaded", "moe_offload_staging_bytes", "moe_offload_workspace_bytes",
           "moe_backward_workspace_bytes", "moe_layer_backward", "moe_layer_forward_keep", "PathShape", "moe_devices_for_expert", "moe_path_count", "moe_path_finalize",
           "moe_path_profile", "moe_popularity_estimate", "moe_schedule_experts",
           "moe_schedule_layer", "moe_top_lists_identical",
           "ACT", "DTYPE", "MoeError", "Shape", "alloc_buffers", "lib", "lib_path",
           "moe_calib_copy", "moe_calib_gemm", "moe_calib_mfma", "moe_capacity", "moe_expert_gemm_kernel", "moe_combine", "moe_dispatch", "moe_dispatch_static",
           "moe_dispatch_static_limit", "moe_expert_ffn",
           "moe_last_error", "moe_layer_chunked", "moe_max_rows", "moe_pack_gate",
           "moe_pack_weights", "moe_packed_gate_bytes", "moe_packed_weight_bytes",
           "moe_profile_enable", "moe_profile_read", "moe_route", "moe_tune_ffn_group_rows",
           "moe_workspace_bytes",
           "STAGES"]
