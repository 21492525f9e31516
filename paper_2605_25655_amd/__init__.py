"""thi: fp16 linear operators of a Llama decoder layer on MI355X (gfx950).

Thin Python binding over the C-ABI library ``libthi.so`` (hand-written HIP
kernels).  The binding only marshals arguments; importing this package does
not import torch or load the library until an operator is called.
"""
from .binding import (  # noqa: F401
    THI_ERR_TIMEOUT,
    THI_ERR_WORKSPACE,
    THI_OK,
    ThiError,
    Workspace,
    library_path,
    load_library,
    thi_attention_workspace_bytes,
    thi_debug_handover,
    thi_decode_attention,
    thi_linear,
    thi_linear_residual,
    thi_linear_static,
    thi_probe_mfma_f16,
    thi_probe_stream_read,
    thi_query_kernel_family,
    thi_rmsnorm_qkv,
    thi_rmsnorm_qkv_rope,
    thi_rmsnorm_swiglu_mlp,
    thi_set_kernel_family,
    thi_set_mlp_fusion,
    thi_set_rowblock_split,
    thi_swiglu_gate_up,
    thi_swiglu_mlp,
    thi_status_string,
    thi_version,
    thi_workspace_bytes,
    thi_workspace_init,
    thi_workspace_status,
)

__all__ = [
    "THI_ERR_TIMEOUT", "THI_ERR_WORKSPACE", "THI_OK", "ThiError", "Workspace", "library_path", "load_library", "thi_attention_workspace_bytes", "thi_decode_attention", "thi_linear", "thi_linear_residual", "thi_linear_static", "thi_probe_mfma_f16", "thi_probe_stream_read", "thi_query_kernel_family",
    "thi_rmsnorm_qkv", "thi_rmsnorm_qkv_rope", "thi_rmsnorm_swiglu_mlp", "thi_set_kernel_family", "thi_set_mlp_fusion", "thi_set_rowblock_split", "thi_swiglu_gate_up", "thi_swiglu_mlp", "thi_status_string", "thi_version",
    "thi_workspace_bytes", "thi_workspace_init", "thi_workspace_status", "thi_debug_handover",
]
