"""Helpers for the GPU parity tests (test infrastructure): move seeded host
arrays to the device, call the library through its binding, bring results back."""
from __future__ import annotations

import sys

import numpy as np


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def to_dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)


def to_host(t) -> np.ndarray:
    import torch
    torch.cuda.synchronize()
    return t.view(torch.int16).cpu().numpy().view(np.float16)


def new_out(M: int, N: int, fill: float = float("nan")):
    import torch
    return torch.full((M, N), fill, dtype=torch.float16, device="cuda")


class Runner:
    """Owns one workspace large enough for a set of shapes and runs the three operators."""

    def __init__(self, M: int, H: int, I: int, n_max: int):
        import paper_2605_25655_amd as thi
        self.thi = thi
        # sized as for more than 32 tokens, so that the tests may force any kernel family (the GEMM kernels
        # need their partial-tile region) on the same workspace at any M
        Mw = max(M, 33)
        need = max(
            thi.thi_workspace_bytes(0, Mw, n_max, max(H, I)),
            thi.thi_workspace_bytes(1, Mw, n_max, max(H, I)),
            thi.thi_workspace_bytes(2, Mw, H, I),
        )
        self.ws = thi.Workspace(need)

    def linear(self, x, w):
        out = new_out(x.shape[0], w.shape[0])
        self.thi.thi_linear(x, w, out, self.ws)
        return out

    def rmsnorm_qkv(self, x, gamma, eps, w):
        out = new_out(x.shape[0], w.shape[0])
        self.thi.thi_rmsnorm_qkv(x, gamma, eps, w, out, self.ws)
        return out

    def swiglu_mlp(self, x, wg, wu, wd):
        out = new_out(x.shape[0], wd.shape[0])
        self.thi.thi_swiglu_mlp(x, wg, wu, wd, out, self.ws)
        return out

    def swiglu_gate_up(self, x, wg, wu):
        out = new_out(x.shape[0], wg.shape[0])
        self.thi.thi_swiglu_gate_up(x, wg, wu, out, self.ws)
        return out

    def linear_residual(self, x, w, res, in_place=False):
        out = res.clone() if in_place else new_out(x.shape[0], w.shape[0])
        self.thi.thi_linear_residual(x, w, out if in_place else res, out, self.ws)
        return out

    def rmsnorm_swiglu_mlp(self, x, gamma, eps, wg, wu, wd, res=None, in_place=False):
        out = res.clone() if (in_place and res is not None) else new_out(x.shape[0], wd.shape[0])
        self.thi.thi_rmsnorm_swiglu_mlp(x, gamma, eps, wg, wu, wd, (out if in_place else res), out, self.ws)
        return out

    def rmsnorm_qkv_rope(self, x, gamma, eps, w, pos, theta, n_rot, head_dim):
        out = new_out(x.shape[0], w.shape[0])
        self.thi.thi_rmsnorm_qkv_rope(x, gamma, eps, w, pos, theta, n_rot, head_dim, out, self.ws)
        return out
