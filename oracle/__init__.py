"""fp64 CPU oracle for the Llama decoder-layer linear operators.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing in the product
package imports it, and it imports nothing from the product package.

The arithmetic lives in ``thi_oracle.c`` (plain C, fp64, index-order loops);
this module only builds that file with gcc and marshals numpy arrays.
Operators follow Sec. III-B.1 (Y = X*W), Sec. III-B.4 (fp16 storage, wider
accumulation and statistics) and Sec. III-C.1 (low-density operators wrapped
around the linear one) of the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "thi_oracle.c")
_LIB = os.path.join(_HERE, "libthi_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile thi_oracle.c into libthi_oracle.so (gcc, OpenMP)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        L = ctypes.c_long
        lib.thi_oracle_threads.restype = ctypes.c_int
        lib.thi_oracle_half_to_double.restype = ctypes.c_double
        lib.thi_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.thi_oracle_silu.restype = ctypes.c_double
        lib.thi_oracle_silu.argtypes = [ctypes.c_double]
        lib.thi_oracle_linear.argtypes = [u16p, u16p, f64p, f64p, L, L, L]
        lib.thi_oracle_rmsnorm_qkv.argtypes = [u16p, u16p, ctypes.c_float, u16p, f64p, f64p, L, L, L]
        lib.thi_oracle_swiglu_mlp.argtypes = [u16p, u16p, u16p, u16p, f64p, f64p, f64p, L, L, L]
        lib.thi_oracle_linear_residual.argtypes = [u16p, u16p, u16p, f64p, f64p, L, L, L]
        lib.thi_oracle_rmsnorm_swiglu_mlp.argtypes = [u16p, u16p, ctypes.c_float, u16p, u16p, u16p, u16p, f64p, f64p,
                                                      f64p, L, L, L]
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.thi_oracle_decode_attention.argtypes = [u16p, u16p, u16p, i32p, ctypes.c_float, f64p, f64p, L, L, L, L, L]
        lib.thi_oracle_rope_inplace.argtypes = [f64p, f64p, i32p, f32p, L, L, L, L]
        lib.thi_oracle_rmsnorm_qkv_rope.argtypes = [u16p, u16p, ctypes.c_float, u16p, i32p, f32p, f64p, f64p,
                                                    L, L, L, L, L]
        _lib = lib
    return _lib


def _bits(a: np.ndarray, shape) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError("oracle inputs are float16 arrays (their bit patterns are read)")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a.view(np.uint16)


def _p16(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _p64(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads() -> int:
    """Number of OpenMP threads the C oracle will use."""
    return int(_load().thi_oracle_threads())


def half_to_double(bits: int) -> float:
    return float(_load().thi_oracle_half_to_double(ctypes.c_uint16(bits)))


def silu(t: float) -> float:
    return float(_load().thi_oracle_silu(ctypes.c_double(t)))


def linear(x: np.ndarray, w: np.ndarray):
    """y[m,n] = sum_k x[m,k] w[n,k] and S[m,n] = sum_k |x[m,k] w[n,k]| in fp64."""
    M, K = x.shape
    N = w.shape[0]
    xb, wb = _bits(x, (M, K)), _bits(w, (N, K))
    y = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)
    rc = _load().thi_oracle_linear(_p16(xb), _p16(wb), _p64(y), _p64(s), M, N, K)
    if rc:
        raise MemoryError("thi_oracle_linear failed")
    return y, s


def rmsnorm_qkv(x: np.ndarray, gamma: np.ndarray, eps: float, w: np.ndarray):
    """y = rmsnorm(x; gamma, eps) w^T and its magnitude sum, in fp64."""
    M, K = x.shape
    N = w.shape[0]
    xb, gb, wb = _bits(x, (M, K)), _bits(gamma, (K,)), _bits(w, (N, K))
    y = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)
    rc = _load().thi_oracle_rmsnorm_qkv(
        _p16(xb), _p16(gb), ctypes.c_float(eps), _p16(wb), _p64(y), _p64(s), M, N, K
    )
    if rc:
        raise MemoryError("thi_oracle_rmsnorm_qkv failed")
    return y, s


def swiglu_mlp(x: np.ndarray, wg: np.ndarray, wu: np.ndarray, wd: np.ndarray, return_h: bool = False):
    """y = (silu(x wg^T) * (x wu^T)) wd^T, S = sum_j |h wd|, optionally h, in fp64."""
    M, H = x.shape
    I = wg.shape[0]
    xb, gb, ub, db = _bits(x, (M, H)), _bits(wg, (I, H)), _bits(wu, (I, H)), _bits(wd, (H, I))
    y = np.empty((M, H), np.float64)
    s = np.empty((M, H), np.float64)
    h = np.empty((M, I), np.float64) if return_h else None
    rc = _load().thi_oracle_swiglu_mlp(
        _p16(xb), _p16(gb), _p16(ub), _p16(db), _p64(y), _p64(s),
        _p64(h) if return_h else None, M, H, I,
    )
    if rc:
        raise MemoryError("thi_oracle_swiglu_mlp failed")
    return (y, s, h) if return_h else (y, s)


def swiglu_gate_up(x: np.ndarray, wg: np.ndarray, wu: np.ndarray):
    """h = silu(x wg^T) * (x wu^T) in fp64 (Sec. III-C.1: the low-density operator behind the gate and up
    projections) and the magnitude S_h that the tolerance 4e-3 * S is taken against for h.

    g = x wg^T and u = x wu^T are two calls of the linear operator, with their magnitude sums S_g, S_u.
    h is not a plain sum of products, so S_h is the first-order image of (S_g, S_u) under
    h(g, u) = silu(g) u:   S_h = |silu'(g) u| S_g + |silu(g)| S_u,   silu'(g) = s (1 + g (1 - s)),
    s = 1 / (1 + exp(-g)) -- an error of eps*S_g in g and eps*S_u in u moves h by eps*S_h to first order."""
    g, sg = linear(x, wg)
    u, su = linear(x, wu)
    sig = 1.0 / (1.0 + np.exp(-g))
    silu_g = g * sig
    dsilu = sig * (1.0 + g * (1.0 - sig))
    h = silu_g * u
    s = np.abs(dsilu * u) * sg + np.abs(silu_g) * su
    return h, s


def linear_residual(x: np.ndarray, w: np.ndarray, res: np.ndarray):
    """y = res + x w^T and S = |res| + sum_k |x w|, in fp64."""
    M, K = x.shape
    N = w.shape[0]
    xb, wb, rb = _bits(x, (M, K)), _bits(w, (N, K)), _bits(res, (M, N))
    y = np.empty((M, N), np.float64)
    s = np.empty((M, N), np.float64)
    rc = _load().thi_oracle_linear_residual(_p16(xb), _p16(wb), _p16(rb), _p64(y), _p64(s), M, N, K)
    if rc:
        raise MemoryError("thi_oracle_linear_residual failed")
    return y, s


def rmsnorm_swiglu_mlp(x, gamma, eps, wg, wu, wd, res=None, return_h: bool = False):
    """y = [res +] (silu(n wg^T) * (n wu^T)) wd^T with n = rmsnorm(x; gamma, eps), in fp64."""
    M, H = x.shape
    I = wg.shape[0]
    xb, gmb = _bits(x, (M, H)), _bits(gamma, (H,))
    gb, ub, db = _bits(wg, (I, H)), _bits(wu, (I, H)), _bits(wd, (H, I))
    rb = _bits(res, (M, H)) if res is not None else None
    y = np.empty((M, H), np.float64)
    s = np.empty((M, H), np.float64)
    h = np.empty((M, I), np.float64) if return_h else None
    rc = _load().thi_oracle_rmsnorm_swiglu_mlp(
        _p16(xb), _p16(gmb), ctypes.c_float(eps), _p16(gb), _p16(ub), _p16(db),
        _p16(rb) if rb is not None else None, _p64(y), _p64(s), _p64(h) if return_h else None, M, H, I)
    if rc:
        raise MemoryError("thi_oracle_rmsnorm_swiglu_mlp failed")
    return (y, s, h) if return_h else (y, s)


def rope_inplace(y: np.ndarray, s, pos: np.ndarray, theta: np.ndarray, n_rot: int, head_dim: int):
    """Rotate the interleaved pairs of the first n_rot columns of y (and the magnitudes s) in place."""
    M, N = y.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    if pos.shape != (M,) or theta.shape != (head_dim // 2,):
        raise ValueError("pos must be [M], theta [head_dim/2]")
    rc = _load().thi_oracle_rope_inplace(
        _p64(y), _p64(s) if s is not None else None,
        pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), theta.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
        M, N, n_rot, head_dim)
    if rc:
        raise ValueError("thi_oracle_rope_inplace: bad arguments")
    return y, s


def rmsnorm_qkv_rope(x, gamma, eps, w, pos, theta, n_rot: int, head_dim: int):
    """rmsnorm_qkv followed by the rotation of the Q and K columns, in fp64."""
    y, s = rmsnorm_qkv(x, gamma, eps, w)
    rope_inplace(y, s, pos, theta, n_rot, head_dim)
    return y, s


def decode_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, seq_lens: np.ndarray, scale: float):
    """y[B,Hq,D] = softmax(scale q k^T) v per head over each request's first seq_lens[b] cached positions
    (q [B,Hq,D]; k, v [B,Hkv,S_max,D]; grouped-query mapping h -> h // (Hq/Hkv)) and S = sum_j p_j |v_j|."""
    B, Hq, D = q.shape
    _, Hkv, S_max, _ = k.shape
    qb, kb, vb = _bits(q, (B, Hq, D)), _bits(k, (B, Hkv, S_max, D)), _bits(v, (B, Hkv, S_max, D))
    lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if lens.shape != (B,):
        raise ValueError("seq_lens must be [B]")
    y = np.empty((B, Hq, D), np.float64)
    s = np.empty((B, Hq, D), np.float64)
    rc = _load().thi_oracle_decode_attention(
        _p16(qb), _p16(kb), _p16(vb), lens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), ctypes.c_float(scale),
        _p64(y), _p64(s), B, Hq, Hkv, D, S_max)
    if rc == -2:
        raise ValueError("thi_oracle_decode_attention: bad arguments")
    if rc:
        raise MemoryError("thi_oracle_decode_attention failed")
    return y, s
