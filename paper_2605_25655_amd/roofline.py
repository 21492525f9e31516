"""Roofline arithmetic used by the benchmark (host only, no device access).

The paper's own analysis (Sec. III-B.1, Eq. 1-3) counts one multiply-accumulate
as one "FLOP" and fp32 operands (4 bytes); its throughput formula (Sec. IV-D,
Eq. 7) does the same and reports units of 2^30.  Those two are kept here exactly
as printed so the tests can pin them to the paper's numbers; everything this
repository reports itself uses 2*M*N*K flops and actual fp16 bytes.
"""
from __future__ import annotations

MI355X_HBM_GBS = 8000.0            # published peak HBM3E bandwidth, GB/s
MI355X_FP16_TFLOPS = 2500.0        # published dense fp16 MFMA peak, TFLOP/s (2.5 PFLOP/s)


def paper_intensity(M: int, K: int, N: int, bytes_per_elem: int = 4) -> float:
    """Eq. 1: MAC count over operand bytes, I = MKN / (b (MK + KN + MN))."""
    return (M * K * N) / (bytes_per_elem * (M * K + K * N + M * N))


def paper_threshold(peak_mac_per_s: float, bandwidth_bytes_per_s: float) -> float:
    """Eq. 2: ridge point of the roofline."""
    return peak_mac_per_s / bandwidth_bytes_per_s


def paper_attainable(peak_mac_per_s: float, bandwidth_bytes_per_s: float, intensity: float) -> float:
    """Eq. 3: P_max = min(peak, B * I)."""
    return min(peak_mac_per_s, bandwidth_bytes_per_s * intensity)


def paper_eq7_gflops(S: int, input_dim: int, output_dim: int, time_ms: float) -> float:
    """Eq. 7 as printed: (S/1024)(in/1024)(out/1024) * 1000/t, i.e. 2^30 MACs per ms-scaled second."""
    return (S / 1024.0) * (input_dim / 1024.0) * (output_dim / 1024.0) * 1000.0 / time_ms


# ---- this repository's conventions -------------------------------------------
def linear_flops(M: int, N: int, K: int) -> float:
    return 2.0 * M * N * K


def linear_bytes(M: int, N: int, K: int, with_gamma: bool = False) -> float:
    """Algorithmic HBM bytes of one projection: weights + activations in + result out (fp16)."""
    return 2.0 * (N * K + M * K + M * N + (K if with_gamma else 0))


def layer_weight_elems(H: int, n_qkv: int, I: int) -> int:
    return n_qkv * H + H * H + 3 * I * H


def layer_bytes(M: int, H: int, n_qkv: int, I: int) -> float:
    """Algorithmic bytes of the three calls of one layer pass (h stays in the workspace and is not counted)."""
    return (linear_bytes(M, n_qkv, H, True) + linear_bytes(M, H, H)
            + 2.0 * (3 * I * H + 2 * M * H))


def layer_flops(M: int, H: int, n_qkv: int, I: int) -> float:
    return 2.0 * M * layer_weight_elems(H, n_qkv, I)
