"""Pins for the oracle's rotary embedding (interleaved pairs, angle = pos * theta[i]).
Expected values come from closed forms, numpy's complex multiplication and invariants."""
import numpy as np
import pytest


def theta_table(head_dim, base=10000.0):
    i = np.arange(head_dim // 2, dtype=np.float64)
    return (base ** (-2.0 * i / head_dim)).astype(np.float32)


def test_position_zero_is_identity(oracle_mod):
    rng = np.random.default_rng(1)
    y = rng.standard_normal((3, 16)); s = np.abs(y) + 1
    y0, s0 = y.copy(), s.copy()
    oracle_mod.rope_inplace(y, s, np.zeros(3, np.int32), theta_table(8), 16, 8)
    assert np.array_equal(y, y0) and np.array_equal(s, s0)


def test_quarter_turn_swaps_pair_with_sign(oracle_mod):
    th = np.array([np.float32(np.pi / 2)], np.float32)          # head_dim 2, one pair
    y = np.array([[3.0, 5.0, 7.0, 11.0]]); s = np.array([[1.0, 2.0, 4.0, 8.0]])
    oracle_mod.rope_inplace(y, s, np.array([1], np.int32), th, 4, 2)
    ang = float(th[0])                                            # fp32(pi/2), widened exactly
    c, sn = np.cos(ang), np.sin(ang)
    np.testing.assert_allclose(y[0], [3 * c - 5 * sn, 5 * c + 3 * sn, 7 * c - 11 * sn, 11 * c + 7 * sn], rtol=1e-15)
    assert abs(y[0, 0] + 5.0) < 1e-6 and abs(y[0, 1] - 3.0) < 1e-6   # (a,b) -> (-b,a)
    np.testing.assert_allclose(s[0], [1 * abs(c) + 2 * sn, 2 * abs(c) + 1 * sn, 4 * abs(c) + 8 * sn, 8 * abs(c) + 4 * sn], rtol=1e-15)


def test_three_quarter_turn_uses_the_magnitude_of_a_negative_sine(oracle_mod):
    """At 3*pi/2 the sine is -1: (a, b) -> (b, -a), and the magnitude map must take |sin| (with the sign kept
    S' would come out negative)."""
    th = np.array([np.float32(np.pi / 2)], np.float32)          # head_dim 2, one pair; position 3
    y = np.array([[3.0, 5.0, 7.0, 11.0]]); s = np.array([[1.0, 2.0, 4.0, 8.0]])
    oracle_mod.rope_inplace(y, s, np.array([3], np.int32), th, 4, 2)
    ang = 3.0 * float(th[0])
    c, sn = np.cos(ang), np.sin(ang)
    assert sn < -0.999999
    np.testing.assert_allclose(y[0], [3 * c - 5 * sn, 5 * c + 3 * sn, 7 * c - 11 * sn, 11 * c + 7 * sn], rtol=1e-15)
    assert abs(y[0, 0] - 5.0) < 1e-5 and abs(y[0, 1] + 3.0) < 1e-5   # (a,b) -> (b,-a)
    np.testing.assert_allclose(s[0], [1 * abs(c) + 2 * abs(sn), 2 * abs(c) + 1 * abs(sn),
                                      4 * abs(c) + 8 * abs(sn), 8 * abs(c) + 4 * abs(sn)], rtol=1e-15)
    assert (s > 0).all() and abs(s[0, 0] - 2.0) < 1e-5 and abs(s[0, 1] - 1.0) < 1e-5


def test_matches_complex_multiplication(oracle_mod):
    rng = np.random.default_rng(2)
    M, heads, d = 5, 3, 8
    N = heads * d + 6                                   # 6 trailing unrotated columns
    y = rng.standard_normal((M, N)); ref = y.copy()
    pos = np.array([0, 1, 7, 100, 4095], np.int32)
    th = theta_table(d)
    oracle_mod.rope_inplace(y, None, pos, th, heads * d, d)
    z = ref[:, :heads * d].reshape(M, heads, d // 2, 2)
    zc = z[..., 0] + 1j * z[..., 1]
    ang = pos[:, None, None].astype(np.float64) * th.astype(np.float64)[None, None, :]
    rot = zc * np.exp(1j * ang)
    exp = np.stack([rot.real, rot.imag], axis=-1).reshape(M, heads * d)
    np.testing.assert_allclose(y[:, :heads * d], exp, rtol=1e-13, atol=1e-13)
    assert np.array_equal(y[:, heads * d:], ref[:, heads * d:])          # V columns untouched


def test_norm_preserved_and_rotations_compose(oracle_mod):
    rng = np.random.default_rng(3)
    d = 16
    y = rng.standard_normal((2, 2 * d)); ref = y.copy()
    th = np.array([2.0 ** -k for k in range(d // 2)], np.float32)        # exactly representable angles
    oracle_mod.rope_inplace(y, None, np.array([3, 5], np.int32), th, 2 * d, d)
    pair_norm = lambda a: (a.reshape(2, -1, 2) ** 2).sum(-1)
    np.testing.assert_allclose(pair_norm(y), pair_norm(ref), rtol=1e-14)
    oracle_mod.rope_inplace(y, None, np.array([4, 2], np.int32), th, 2 * d, d)   # now at positions 7 and 7
    once = ref.copy()
    oracle_mod.rope_inplace(once, None, np.array([7, 7], np.int32), th, 2 * d, d)
    np.testing.assert_allclose(y, once, rtol=1e-13, atol=1e-14)


def test_scores_depend_on_relative_position_only(oracle_mod):
    rng = np.random.default_rng(4)
    d = 8
    q = rng.standard_normal((1, d)); k = rng.standard_normal((1, d))
    th = np.array([2.0 ** -k_ for k_ in range(d // 2)], np.float32)
    def score(pq, pk):
        a, b = q.copy(), k.copy()
        oracle_mod.rope_inplace(a, None, np.array([pq], np.int32), th, d, d)
        oracle_mod.rope_inplace(b, None, np.array([pk], np.int32), th, d, d)
        return float((a * b).sum())
    assert abs(score(10, 3) - score(107, 100)) < 1e-12
    assert abs(score(10, 3) - score(9, 3)) > 1e-3


def test_theta_index_wraps_per_head(oracle_mod):
    """Column c of any head uses theta[(c mod head_dim)/2]: two heads with equal inputs rotate equally."""
    d = 4
    y = np.tile(np.array([[1.0, 2.0, 3.0, 4.0]]), (1, 2))
    oracle_mod.rope_inplace(y, None, np.array([1], np.int32), np.array([0.5, 0.25], np.float32), 2 * d, d)
    assert np.array_equal(y[0, :d], y[0, d:])
    assert abs(y[0, 0] - (np.cos(0.5) - 2 * np.sin(0.5))) < 1e-15
    assert abs(y[0, 2] - (3 * np.cos(0.25) - 4 * np.sin(0.25))) < 1e-15


def test_bad_arguments_rejected(oracle_mod):
    y = np.zeros((1, 8))
    with pytest.raises(ValueError):
        oracle_mod.rope_inplace(y, None, np.zeros(1, np.int32), np.zeros(2, np.float32), 6, 4)   # n_rot % head_dim


def test_fused_entry_equals_projection_then_rotation(oracle_mod):
    from paper_2605_25655_amd import synth
    x, w, g = synth.random_problem(31, 3, 48, 64)
    pos = np.array([0, 5, 77], np.int32); th = theta_table(16)
    y1, s1 = oracle_mod.rmsnorm_qkv_rope(x, g, 1e-6, w, pos, th, 32, 16)
    y2, s2 = oracle_mod.rmsnorm_qkv(x, g, 1e-6, w)
    oracle_mod.rope_inplace(y2, s2, pos, th, 32, 16)
    assert np.array_equal(y1, y2) and np.array_equal(s1, s2)
