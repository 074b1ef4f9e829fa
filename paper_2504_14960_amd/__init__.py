"""MI355X-native MoE-layer forward hot path (arXiv 2504.14960, Section 3.3).

A thin ctypes binding over ``libmoe_hip.so``; every step of the path (router,
permute, grouped SwiGLU expert GEMMs, un-permute/combine) runs in the HIP
kernels of ``csrc/``.  PyTorch is used for device memory and streams only.
"""
from .binding import (  # noqa: F401
    MOE_BF16,
    MOE_F32,
    MoeError,
    capacity_from_factor,
    expert_backward_workspace_bytes,
    expert_down,
    expert_down_fp8,
    expert_gate_up,
    expert_gate_up_fp8,
    expert_weights_transpose,
    fp8_delayed_scale,
    fp8_quantize,
    grouped_gemm_swiglu,
    grouped_gemm_swiglu_backward,
    grouped_gemm_swiglu_fp8,
    layer_forward,
    layer_workspace_bytes,
    layer_workspace_layout,
    lib,
    lib_path,
    max_rows,
    permute,
    permute_backward,
    permute_fp8,
    permute_workspace_bytes,
    router_topk,
    set_option,
    unpermute_combine,
    unpermute_combine_backward,
    version,
)
