"""Seeded synthetic inputs for the Llama decoder-layer linear operators.

This module holds NO arithmetic of the method: it only names the five layer
shapes and draws random fp16 tensors.  It is the one module that both the GPU
tests and the CPU oracle's tests may share.

The shapes are the Llama-2 7B/13B/30B/70B layer shapes the paper evaluates on
(Sec. IV-A, model list) plus a tiny layer; the paper's data set is itself a
synthetic, length-padded prompt set, so random tensors of the right shape and
spread stand in for trained weights and real activations.

Recipe (per config c = 1..5): rng = Generator(Philox(key=20260525 + c)); draw,
in this fixed order, float64 standard normals scaled and cast to fp16 (RNE):
w_qkv [N_qkv,H]*sigma, w_o [H,H]*sigma, w_gate [I,H]*sigma, w_up [I,H]*sigma,
w_down [H,I]*sigma, gamma [H] = 1 + 0.1*z; then for every M of the config, in
list order: x_qkv [M,H], a_o [M,H], x_mlp [M,H] ~ N(0,1).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

SEED_BASE = 20260525
EPS = 1e-6


@dataclass(frozen=True)
class LayerConfig:
    index: int
    name: str
    hidden: int          # H
    n_qkv: int           # rows of the stacked Wq;Wk;Wv
    inter: int           # I
    sigma_w: float
    decode_m: Tuple[int, ...]
    prefill_m: Tuple[int, ...]

    @property
    def weight_elems(self) -> int:
        H, I = self.hidden, self.inter
        return self.n_qkv * H + H * H + 3 * I * H

    @property
    def all_m(self) -> Tuple[int, ...]:
        return tuple(self.decode_m) + tuple(self.prefill_m)


CONFIGS: Dict[int, LayerConfig] = {
    1: LayerConfig(1, "tiny", 512, 1536, 1376, 0.02, (1,), ()),
    2: LayerConfig(2, "llama-7b", 4096, 12288, 11008, 0.02, (1, 8, 32), ()),
    3: LayerConfig(3, "llama-13b", 5120, 15360, 13824, 0.02, (16,), (512,)),
    4: LayerConfig(4, "llama-30b", 6656, 19968, 17920, 0.02, (32,), (1024, 2048)),
    5: LayerConfig(5, "llama-70b-gqa", 8192, 10240, 28672, 0.015, (1, 32), (2048,)),
}


def _normal_f16(rng: np.random.Generator, shape, scale: float = 1.0, shift: float = 0.0,
                chunk_rows: int = 2048) -> np.ndarray:
    """float64 standard normals * scale + shift, cast to fp16; drawn in row chunks
    (same stream as one big draw) so the fp64 temporary stays small."""
    out = np.empty(shape, np.float16)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(1, -1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        z = rng.standard_normal((r1 - r0, flat.shape[1]))
        flat[r0:r1] = (z * scale + shift).astype(np.float16)
    return out


def layer_rng(cfg: LayerConfig) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=SEED_BASE + cfg.index))


def make_layer(cfg: LayerConfig, ms=None) -> dict:
    """All tensors of one config as host numpy fp16 arrays.

    Returns {"w_qkv","w_o","w_gate","w_up","w_down","gamma","eps",
             "acts": {M: {"x_qkv","a_o","x_mlp"}}}.  Activations are always drawn
    for every M of the config, in order (so a given M sees the same values no
    matter which subset ``ms`` is kept)."""
    rng = layer_rng(cfg)
    H, I, s = cfg.hidden, cfg.inter, cfg.sigma_w
    out = {
        "w_qkv": _normal_f16(rng, (cfg.n_qkv, H), s),
        "w_o": _normal_f16(rng, (H, H), s),
        "w_gate": _normal_f16(rng, (I, H), s),
        "w_up": _normal_f16(rng, (I, H), s),
        "w_down": _normal_f16(rng, (H, I), s),
        "gamma": _normal_f16(rng, (H,), 0.1, 1.0),
        "eps": EPS,
        "acts": {},
    }
    for M in cfg.all_m:
        acts = {
            "x_qkv": _normal_f16(rng, (M, H)),
            "a_o": _normal_f16(rng, (M, H)),
            "x_mlp": _normal_f16(rng, (M, H)),
        }
        if ms is None or M in ms:
            out["acts"][M] = acts
    return out


def random_problem(seed: int, M: int, N: int, K: int, sigma_w: float = 0.02):
    """One free-form (x[M,K], w[N,K], gamma[K]) triple for odd-shape parity cases."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    w = _normal_f16(rng, (N, K), sigma_w)
    x = _normal_f16(rng, (M, K))
    gamma = _normal_f16(rng, (K,), 0.1, 1.0)
    return x, w, gamma


def sample_rows(seed: int, M: int, count: int = 32) -> np.ndarray:
    """Deterministic row subset for prefill-size checks: tile-edge rows plus
    seeded random rows, sorted, unique, ``count`` of them (or all rows if M is
    smaller)."""
    if M <= count:
        return np.arange(M)
    fixed = [0, 1, 127, 128, 255, 256, M // 2 - 1, M // 2, M - 2, M - 1]
    rows = sorted({r for r in fixed if 0 <= r < M})
    rng = np.random.Generator(np.random.Philox(key=seed))
    while len(rows) < count:
        r = int(rng.integers(0, M))
        if r not in rows:
            rows.append(r)
    return np.array(sorted(rows))
