"""ctypes binding over libthi.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device memory; every
arithmetic step runs in the HIP kernels behind the C ABI (include/thi.h).
There is no CPU fallback: if the library is missing or was not built, calls
raise.
"""
from __future__ import annotations

import ctypes
import os

THI_OK = 0
THI_ERR_WORKSPACE = 4
THI_ERR_TIMEOUT = 6
THI_OP_RMSNORM_QKV, THI_OP_LINEAR, THI_OP_SWIGLU_MLP = 0, 1, 2

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libthi.so")
_PROBE_LIB_PATH = os.path.join(_PKG, "libthi_probe.so")
_lib = None
_probe_lib = None

EXPORTED_SYMBOLS = (
    "thi_rmsnorm_qkv", "thi_rmsnorm_qkv_rope", "thi_linear", "thi_linear_static", "thi_swiglu_mlp", "thi_swiglu_gate_up",
    "thi_linear_residual", "thi_rmsnorm_swiglu_mlp", "thi_decode_attention", "thi_attention_workspace_bytes",
    "thi_workspace_bytes",
    "thi_workspace_init", "thi_workspace_status", "thi_debug_handover", "thi_status_string", "thi_version", "thi_set_kernel_family", "thi_set_rowblock_split", "thi_set_mlp_fusion", "thi_query_kernel_family",
)
# the benchmark's measurement probes live in a library of their own (include/thi_probe.h)
PROBE_SYMBOLS = ("thi_probe_stream_read", "thi_probe_mfma_f16")


class ThiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {thi_status_string(status)} (status {status})")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libthi.so (built in-tree by ``python -m paper_2605_25655_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2605_25655_amd.build` "
            "(there is no fallback path)")
    # The tensors and streams handed to the library belong to the HIP runtime that PyTorch loaded;
    # libthi must bind to that same copy of the runtime, so PyTorch's is loaded first.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, ci, cf = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
    lib.thi_rmsnorm_qkv.argtypes = [vp, vp, cf, vp, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_rmsnorm_qkv.restype = ci
    lib.thi_rmsnorm_qkv_rope.argtypes = [vp, vp, cf, vp, vp, vp, ci, ci, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_rmsnorm_qkv_rope.restype = ci
    lib.thi_linear.argtypes = [vp, vp, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_linear.restype = ci
    lib.thi_linear_static.argtypes = [vp, vp, vp, ci, ci, ci, vp]
    lib.thi_linear_static.restype = ci
    lib.thi_swiglu_mlp.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_swiglu_mlp.restype = ci
    lib.thi_swiglu_gate_up.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_swiglu_gate_up.restype = ci
    lib.thi_linear_residual.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_linear_residual.restype = ci
    lib.thi_rmsnorm_swiglu_mlp.argtypes = [vp, vp, cf, vp, vp, vp, vp, vp, ci, ci, ci, vp, sz, vp]
    lib.thi_rmsnorm_swiglu_mlp.restype = ci
    lib.thi_decode_attention.argtypes = [vp, vp, vp, vp, cf, vp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.thi_decode_attention.restype = ci
    lib.thi_attention_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.thi_attention_workspace_bytes.restype = sz
    lib.thi_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.thi_workspace_bytes.restype = sz
    lib.thi_workspace_init.argtypes = [vp, sz, vp]
    lib.thi_workspace_init.restype = ci
    lib.thi_workspace_status.argtypes = [vp, sz, vp]
    lib.thi_workspace_status.restype = ci
    lib.thi_debug_handover.argtypes = [ctypes.c_uint, ci]
    lib.thi_debug_handover.restype = ci
    lib.thi_status_string.argtypes = [ci]
    lib.thi_status_string.restype = ctypes.c_char_p
    lib.thi_version.argtypes = []
    lib.thi_version.restype = ci
    lib.thi_query_kernel_family.argtypes = [ci, ci, ci, ci]
    lib.thi_query_kernel_family.restype = ci
    lib.thi_set_kernel_family.argtypes = [ci]
    lib.thi_set_kernel_family.restype = ci
    lib.thi_set_mlp_fusion.argtypes = [ci]
    lib.thi_set_mlp_fusion.restype = ci
    lib.thi_set_rowblock_split.argtypes = [ci]
    lib.thi_set_rowblock_split.restype = ci
    _lib = lib
    return lib


def thi_status_string(status: int) -> str:
    return load_library().thi_status_string(int(status)).decode()


def thi_version() -> int:
    return int(load_library().thi_version())


def thi_workspace_bytes(op: int, M: int, N_or_H: int, K_or_I: int) -> int:
    return int(load_library().thi_workspace_bytes(int(op), int(M), int(N_or_H), int(K_or_I)))


def thi_query_kernel_family(M: int, N: int, K: int, fused: int = 0) -> int:
    """1 = stream-K decode kernel, 2 = MFMA GEMM, 3 = row-slab decode kernel, 4 = row-block decode kernel
    (what a call would run)."""
    return int(load_library().thi_query_kernel_family(int(M), int(N), int(K), int(fused)))


def thi_set_kernel_family(family: int) -> int:
    return int(load_library().thi_set_kernel_family(int(family)))


def thi_set_mlp_fusion(on: bool) -> int:
    """Opt-in: the decode MLP as one launch where the library has that kernel (default off); returns the previous setting."""
    return int(load_library().thi_set_mlp_fusion(int(bool(on))))


def thi_set_rowblock_split(split: int) -> int:
    return int(load_library().thi_set_rowblock_split(int(split)))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


class Workspace:
    """A caller-owned workspace: a torch byte tensor plus the one-time init call."""

    def __init__(self, nbytes: int, device="cuda", stream=None, init: bool = True):
        """init=False: for thi_decode_attention alone, whose workspace needs no preparation."""
        import torch
        self.nbytes = int(nbytes)
        self.buffer = torch.empty(self.nbytes + 256, dtype=torch.uint8, device=device)
        off = (-self.buffer.data_ptr()) % 256
        self.ptr = self.buffer.data_ptr() + off
        if init:
            thi_workspace_init(self.ptr, self.nbytes, stream)

    def reinit(self, stream=None) -> None:
        thi_workspace_init(self.ptr, self.nbytes, stream)

    @classmethod
    def for_ops(cls, shapes, device="cuda", stream=None):
        """shapes: iterable of (op, M, N_or_H, K_or_I); sized for the largest."""
        need = max(thi_workspace_bytes(*s) for s in shapes)
        return cls(need, device=device, stream=stream)


def _ws(workspace):
    if isinstance(workspace, Workspace):
        return ctypes.c_void_p(workspace.ptr), workspace.nbytes
    ptr, nbytes = workspace
    return ctypes.c_void_p(int(ptr)), int(nbytes)


def thi_workspace_init(ptr: int, nbytes: int, stream=None) -> None:
    rc = load_library().thi_workspace_init(ctypes.c_void_p(int(ptr)), int(nbytes), _stream(stream))
    if rc != THI_OK:
        raise ThiError(rc, "thi_workspace_init")


def thi_workspace_status(workspace, stream=None) -> int:
    """THI_OK, or THI_ERR_TIMEOUT if a hand-over timed out on this workspace since its last init (waits for the stream)."""
    wp, wb = _ws(workspace)
    return int(load_library().thi_workspace_status(wp, wb, _stream(stream)))


def thi_debug_handover(spin_limit: int, withhold_flags: bool) -> None:
    """Test hook: force the stream-K hand-over's bounded wait to run out (0, False restores the defaults)."""
    load_library().thi_debug_handover(int(spin_limit), int(bool(withhold_flags)))


def thi_rmsnorm_qkv(x, gamma, eps: float, w_qkv, out, workspace, stream=None, check: bool = True) -> int:
    """out[M,N] = rmsnorm(x[M,K]; gamma[K], eps) @ w_qkv[N,K]^T  (fp16 device tensors)."""
    M, K = x.shape
    N = w_qkv.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_rmsnorm_qkv(_ptr(x), _ptr(gamma), float(eps), _ptr(w_qkv), _ptr(out),
                                        M, N, K, wp, wb, _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_rmsnorm_qkv")
    return rc


def thi_linear(x, w, out, workspace, stream=None, check: bool = True) -> int:
    """out[M,N] = x[M,K] @ w[N,K]^T  (fp16 device tensors)."""
    M, K = x.shape
    N = w.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_linear(_ptr(x), _ptr(w), _ptr(out), M, N, K, wp, wb, _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_linear")
    return rc


def thi_linear_static(x, w, out, stream=None, check: bool = True) -> int:
    """out[M,N] = x[M,K] @ w[N,K]^T for M <= 32, on the library's static scratch array (nothing is allocated)."""
    M, K = x.shape
    N = w.shape[0]
    rc = load_library().thi_linear_static(_ptr(x), _ptr(w), _ptr(out), M, N, K, _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_linear_static")
    return rc


def thi_swiglu_mlp(x, w_gate, w_up, w_down, out, workspace, stream=None, check: bool = True) -> int:
    """out[M,H] = (silu(x @ w_gate^T) * (x @ w_up^T)) @ w_down^T  (fp16 device tensors)."""
    M, H = x.shape
    I = w_gate.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_swiglu_mlp(_ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out),
                                       M, H, I, wp, wb, _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_swiglu_mlp")
    return rc


def thi_linear_residual(x, w, residual, out, workspace, stream=None, check: bool = True) -> int:
    """out[M,N] = residual[M,N] + x[M,K] @ w[N,K]^T  (fp16 device tensors; residual may be out)."""
    M, K = x.shape
    N = w.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_linear_residual(_ptr(x), _ptr(w), _ptr(residual), _ptr(out), M, N, K, wp, wb,
                                            _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_linear_residual")
    return rc


def thi_rmsnorm_swiglu_mlp(x, gamma, eps, w_gate, w_up, w_down, residual, out, workspace, stream=None,
                           check: bool = True) -> int:
    """out[M,H] = [residual +] (silu(n @ w_gate^T) * (n @ w_up^T)) @ w_down^T, n = rmsnorm(x; gamma, eps)."""
    M, H = x.shape
    I = w_gate.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_rmsnorm_swiglu_mlp(_ptr(x), _ptr(gamma), ctypes.c_float(eps), _ptr(w_gate), _ptr(w_up),
                                               _ptr(w_down), _ptr(residual), _ptr(out), M, H, I, wp, wb,
                                               _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_rmsnorm_swiglu_mlp")
    return rc


def thi_attention_workspace_bytes(B: int, Hq: int, Hkv: int, D: int, S_max: int) -> int:
    return int(load_library().thi_attention_workspace_bytes(int(B), int(Hq), int(Hkv), int(D), int(S_max)))


def thi_decode_attention(q, k_cache, v_cache, seq_lens, scale, out, workspace, stream=None, check: bool = True) -> int:
    """out[B,Hq,D] = softmax(scale q k^T) v per head over each request's first seq_lens[b] cached positions.

    q, out [B,Hq,D]; k_cache, v_cache [B,Hkv,S_max,D] fp16 device tensors; seq_lens [B] int32 device tensor."""
    B, Hq, D = q.shape
    _, Hkv, S_max, _ = k_cache.shape
    wp, wb = _ws(workspace)
    rc = load_library().thi_decode_attention(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), ctypes.c_float(scale),
                                             _ptr(out), B, Hq, Hkv, D, S_max, wp, wb, _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_decode_attention")
    return rc


def thi_swiglu_gate_up(x, w_gate, w_up, h, workspace, stream=None, check: bool = True) -> int:
    """h[M,I] = silu(x @ w_gate^T) * (x @ w_up^T)  (fp16 device tensors)."""
    M, H = x.shape
    I = w_gate.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_swiglu_gate_up(_ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(h), M, H, I, wp, wb,
                                           _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_swiglu_gate_up")
    return rc


def probe_library_path() -> str:
    return _PROBE_LIB_PATH


def load_probe_library():
    """Load libthi_probe.so (the benchmark's measurement probes; built next to libthi.so)."""
    global _probe_lib
    if _probe_lib is not None:
        return _probe_lib
    if not os.path.exists(_PROBE_LIB_PATH):
        raise FileNotFoundError(f"{_PROBE_LIB_PATH} is missing: build it with `python -m paper_2605_25655_amd.build`")
    import torch  # noqa: F401  (the same copy of the HIP runtime as the tensors', see load_library)
    lib = ctypes.CDLL(_PROBE_LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.thi_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.thi_probe_stream_read.restype = ci
    lib.thi_probe_mfma_f16.argtypes = [vp, ci, ci, vp, vp]
    lib.thi_probe_mfma_f16.restype = ci
    _probe_lib = lib
    return lib


def thi_probe_stream_read(buffer, sink, stream=None) -> None:
    """Enqueue one streaming read of `buffer` (device tensor, >= 16 MiB)."""
    rc = load_probe_library().thi_probe_stream_read(_ptr(buffer), buffer.numel() * buffer.element_size(), _ptr(sink),
                                              _stream(stream))
    if rc != THI_OK:
        raise ThiError(rc, "thi_probe_stream_read")


def thi_probe_mfma_f16(operands, iters: int, workgroups: int, sink, stream=None) -> float:
    """Enqueue the register-only MFMA loop; returns the flops it performs."""
    rc = load_probe_library().thi_probe_mfma_f16(_ptr(operands), int(iters), int(workgroups), _ptr(sink), _stream(stream))
    if rc != THI_OK:
        raise ThiError(rc, "thi_probe_mfma_f16")
    return float(workgroups) * 8 * iters * 8 * 32768.0


def thi_rmsnorm_qkv_rope(x, gamma, eps: float, w_qkv, positions, theta, n_rot: int, head_dim: int, out, workspace,
                         stream=None, check: bool = True) -> int:
    """thi_rmsnorm_qkv with rotary embedding on columns [0, n_rot): positions int32 [M], theta fp32 [head_dim/2]."""
    M, K = x.shape
    N = w_qkv.shape[0]
    wp, wb = _ws(workspace)
    rc = load_library().thi_rmsnorm_qkv_rope(_ptr(x), _ptr(gamma), float(eps), _ptr(w_qkv), _ptr(positions),
                                             _ptr(theta), int(n_rot), int(head_dim), _ptr(out), M, N, K, wp, wb,
                                             _stream(stream))
    if check and rc != THI_OK:
        raise ThiError(rc, "thi_rmsnorm_qkv_rope")
    return rc
