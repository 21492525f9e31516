"""The roofline helpers restate Eq. 1-3 and Eq. 7; the expected values are the
ones the paper prints (tests/golden/*.txt)."""
import os
from fractions import Fraction

from paper_2605_25655_amd import roofline

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kv(path):
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_eq1_to_eq3_match_printed_analysis():
    g = _kv(os.path.join(GOLD, "paper_roofline.txt"))
    I = roofline.paper_intensity(int(g["tile_M"]), int(g["tile_K"]), int(g["tile_N"]))
    assert Fraction(I).limit_denominator(1000) == Fraction(int(g["intensity_num"]), int(g["intensity_den"]))
    thr = roofline.paper_threshold(g["peak_mac_per_s"], g["bandwidth_gbs"] * 1e9)
    assert abs(thr - g["threshold"]) < 1e-9
    # the chosen tile sits far below the ridge -> bandwidth-bound, attainable = B*I
    assert roofline.paper_attainable(g["peak_mac_per_s"], g["bandwidth_gbs"] * 1e9, I) == g["bandwidth_gbs"] * 1e9 * I
    assert roofline.paper_attainable(g["peak_mac_per_s"], g["bandwidth_gbs"] * 1e9, 1e6) == g["peak_mac_per_s"]


def test_eq7_reproduces_printed_throughput():
    for line in open(os.path.join(GOLD, "paper_linear_table.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        S, kin, kout, _prec, ms, printed, frac, peak = line.split()
        val = roofline.paper_eq7_gflops(int(S), int(kin), int(kout), float(ms))
        # the printed figure converts 2^30 to 1e9
        assert abs(val * 2 ** 30 / 1e9 - float(printed)) < 0.01 * 1.0 + 0.5
        assert abs(val * 2 ** 30 / 1e9 / float(peak) - float(frac)) < 1e-3


def test_layer_byte_counts_match_config_table():
    from paper_2605_25655_amd import synth
    expect = {1: 3162112, 2: 202375168, 3: 317194240, 4: 535035904, 5: 855638016}
    for i, cfg in synth.CONFIGS.items():
        assert cfg.weight_elems == expect[i]
        assert roofline.layer_weight_elems(cfg.hidden, cfg.n_qkv, cfg.inter) == expect[i]
    c = synth.CONFIGS[2]
    assert abs(roofline.layer_bytes(1, c.hidden, c.n_qkv, c.inter) / 1e6 - 404.75) < 0.1
