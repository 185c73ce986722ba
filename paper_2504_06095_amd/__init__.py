"""MI355X-native shard hot path of Nonuniform Tensor Parallelism (arXiv 2504.06095).

The product is libntp.so (HIP kernels behind the C ABI of include/ntp.h); `binding`
marshals arguments to it and `inputs` makes seeded synthetic data.  Importing the
package loads nothing; the first call into `binding` loads the library and raises
if it has not been built.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    NtpError, ReshardPlan, attn_core_shape, ntp_attn_core_shard_fwd, ntp_attn_core_shard_bwd, ntp_attn_core_choice, ntp_reshard_row_segments, row_segments, ntp_mlp_shard_bwd_resharded,
    ntp_attn_proj_shard_bwd_resharded, ntp_comp_sync_plan, ntp_gemm_choice, ntp_reshard_plan_create, ntp_attn_proj_shard_bwd, ntp_attn_proj_shard_fwd, ntp_attn_shard_plan, ntp_calibration_copy,
    ntp_kernel_timing_enable, ntp_kernel_timing_read, ntp_mlp_shard_bwd,
    ntp_mlp_shard_fwd, ntp_reshard_grad, ntp_reshard_segments, ntp_set_workspace, ntp_shard_plan, ntp_version, tensor_spec,
    Handle, default_handle, ntp_create, ntp_destroy, ntp_device_info, ntp_set_option, ntp_workspace_bytes, ntp_attn_proj_shard_fwd_static, ntp_replica_sum, ntp_probe_rates,
)
