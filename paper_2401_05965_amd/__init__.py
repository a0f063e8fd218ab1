"""libhap: MI355X-native per-device compute of HAP-style unevenly sharded SPMD programs.

The package is a thin ctypes binding over the C-ABI library ``libhap.so`` built from
``csrc/`` (see ``include/libhap.h`` for the contract).  PyTorch appears only as the owner
of device memory and streams; every arithmetic step runs in the library's kernels.
"""
from .binding import (  # noqa: F401
    HapError, LinearDesc, AttnDesc, MoeDesc, GatherDesc, Stage, lib, lib_path,
    F32, BF16, SHARD_BATCH, SHARD_FEATURE, SHARD_REDUCTION, REPLICATED, ACT_NONE, ACT_GELU_ERF,
    hap_shard_ratios, hap_iteration_time, hap_round_shards, hap_shard_ratios_segments, hap_iteration_time_segments, hap_synthesize, hap_program_time, hap_program_stages, hap_optimize,
    hap_version, hap_strerror, hap_last_error,
    hap_sharded_linear_fwd, hap_sharded_linear_bwd, hap_sharded_linear_bwd_dact, hap_linear_fwd_workspace, hap_linear_bwd_workspace,
    hap_sfb_grad, hap_sfb_grad_static, hap_sfb_workspace, hap_sharded_attn_fwd, hap_sharded_attn_bwd, hap_attn_bwd_workspace,
    hap_layernorm_fwd, hap_layernorm_bwd, hap_layernorm_bwd_workspace,
    hap_moe_linear_fwd, hap_moe_linear_bwd, hap_moe_linear_bwd_dact, hap_moe_linear_fwd_workspace, hap_moe_linear_bwd_workspace,
    hap_allgather_capacity, hap_allgather_pad, hap_allgather_assemble, hap_reducescatter_split,
    hap_gelu_bwd, hap_add, hap_colsum, hap_colsum_workspace, hap_probe_mfma_bf16, hap_debug_set_gemm_view_limit, hap_device_info,
)
