"""Pins for the decode-attention oracle (Eq. 6 per head, per request, grouped-query mapping).

Fixed against closed forms, an independent library routine (scipy's softmax with numpy contractions on
exactly widened inputs) and structural facts; each is chosen so that a plausible slip -- a missing scale,
a transposed cache, the wrong key/value head, positions past the request's length -- fails."""
import numpy as np
import pytest
from scipy.special import softmax


def f16(a):
    return np.asarray(a, dtype=np.float16)


def test_single_position_returns_its_value_row(oracle_mod):
    rng = np.random.default_rng(1)
    B, Hq, Hkv, D, S = 2, 4, 2, 8, 5
    q, k, v = f16(rng.standard_normal((B, Hq, D))), f16(rng.standard_normal((B, Hkv, S, D))), f16(rng.standard_normal((B, Hkv, S, D)))
    y, s = oracle_mod.decode_attention(q, k, v, np.array([1, 1]), 0.37)
    for b in range(B):
        for h in range(Hq):
            assert np.array_equal(y[b, h], v[b, h // 2, 0].astype(np.float64))
            assert np.array_equal(s[b, h], np.abs(v[b, h // 2, 0].astype(np.float64)))


def test_zero_query_gives_the_mean_of_the_live_rows_only(oracle_mod):
    rng = np.random.default_rng(2)
    B, H, D, S = 3, 2, 16, 12
    k, v = f16(rng.standard_normal((B, H, S, D))), f16(rng.standard_normal((B, H, S, D)))
    lens = np.array([12, 5, 1])
    y, _ = oracle_mod.decode_attention(f16(np.zeros((B, H, D))), k, v, lens, 1.0)
    for b in range(B):
        want = v[b, :, : lens[b]].astype(np.float64).mean(axis=1)
        np.testing.assert_allclose(y[b], want, rtol=1e-14, atol=1e-15)


def test_zero_length_request_gives_zero(oracle_mod):
    rng = np.random.default_rng(3)
    q, k, v = f16(rng.standard_normal((2, 2, 8))), f16(rng.standard_normal((2, 2, 4, 8))), f16(rng.standard_normal((2, 2, 4, 8)))
    y, s = oracle_mod.decode_attention(q, k, v, np.array([0, 3]), 1.0)
    assert not y[0].any() and not s[0].any() and y[1].any()


def test_two_positions_closed_form_checks_the_scale(oracle_mod):
    # scores t0 = scale * 4, t1 = 0: p0 = 1 / (1 + exp(-4 scale)); value rows 1 and -1
    D = 4
    q = f16(np.ones((1, 1, D)))
    k = f16(np.zeros((1, 1, 2, D)))
    k[0, 0, 0] = 1.0
    v = f16(np.zeros((1, 1, 2, D)))
    v[0, 0, 0], v[0, 0, 1] = 1.0, -1.0
    for scale in (0.5, 1.0 / np.sqrt(D), 2.0):
        sc = float(np.float32(scale))
        y, s = oracle_mod.decode_attention(q, k, v, np.array([2]), sc)
        p0 = 1.0 / (1.0 + np.exp(-4.0 * sc))
        np.testing.assert_allclose(y[0, 0], np.full(D, 2 * p0 - 1), rtol=1e-14)
        np.testing.assert_allclose(s[0, 0], np.ones(D), rtol=1e-14)


def test_dominant_key_selects_its_value(oracle_mod):
    # one key lines up with the query so strongly that every other weight underflows to nothing
    rng = np.random.default_rng(4)
    D, S = 8, 9
    q = f16(np.full((1, 1, D), 8.0))
    k = f16(rng.uniform(-0.1, 0.1, (1, 1, S, D)))
    k[0, 0, 6] = 8.0
    v = f16(rng.standard_normal((1, 1, S, D)))
    y, _ = oracle_mod.decode_attention(q, k, v, np.array([S]), 4.0)
    np.testing.assert_allclose(y[0, 0], v[0, 0, 6].astype(np.float64), rtol=1e-12, atol=1e-300)


def test_shift_of_all_scores_changes_nothing(oracle_mod):
    # the first d component of every key carries the same offset c: scores shift by scale*q0*c, weights do not
    rng = np.random.default_rng(5)
    B, H, D, S = 1, 2, 8, 7
    q = f16(rng.standard_normal((B, H, D)))
    k = f16(rng.standard_normal((B, H, S, D)))
    v = f16(rng.standard_normal((B, H, S, D)))
    k0 = k.copy()
    k0[..., 0] = 0.0
    k1 = k0.copy()
    k1[..., 0] = 2.0            # exact in fp16
    y0, _ = oracle_mod.decode_attention(q, k0, v, np.array([S]), 0.5)
    y1, _ = oracle_mod.decode_attention(q, k1, v, np.array([S]), 0.5)
    np.testing.assert_allclose(y0, y1, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("B,Hq,Hkv,D,S", [(2, 4, 4, 16, 33), (3, 8, 2, 32, 50), (1, 16, 2, 64, 129)])
def test_library_witness_with_ragged_lengths_and_grouped_heads(oracle_mod, B, Hq, Hkv, D, S):
    rng = np.random.default_rng(10 + B + Hq + D)
    q, k, v = f16(rng.standard_normal((B, Hq, D))), f16(rng.standard_normal((B, Hkv, S, D))), f16(rng.standard_normal((B, Hkv, S, D)))
    lens = rng.integers(1, S + 1, size=B)
    lens[0] = S
    scale = float(np.float32(1.0 / np.sqrt(D)))
    y, s = oracle_mod.decode_attention(q, k, v, lens, scale)
    G = Hq // Hkv
    for b in range(B):
        L = lens[b]
        for h in range(Hq):
            kk, vv = k[b, h // G, :L].astype(np.float64), v[b, h // G, :L].astype(np.float64)
            p = softmax(scale * (kk @ q[b, h].astype(np.float64)))
            np.testing.assert_allclose(y[b, h], p @ vv, rtol=1e-12, atol=1e-14)
            np.testing.assert_allclose(s[b, h], p @ np.abs(vv), rtol=1e-12, atol=1e-14)


def test_grouped_query_heads_share_the_right_cache_head(oracle_mod):
    # Hq = 4, Hkv = 2: heads 0,1 -> cache head 0, heads 2,3 -> cache head 1 (not h % Hkv)
    D, S = 8, 3
    q = f16(np.zeros((1, 4, D)))
    k = f16(np.zeros((1, 2, S, D)))
    v = f16(np.zeros((1, 2, S, D)))
    v[0, 0], v[0, 1] = 1.0, 5.0
    y, _ = oracle_mod.decode_attention(q, k, v, np.array([S]), 1.0)
    assert np.array_equal(y[0, :, 0], np.array([1.0, 1.0, 5.0, 5.0]))


def test_bad_arguments(oracle_mod):
    q, k = f16(np.zeros((1, 3, 8))), f16(np.zeros((1, 2, 4, 8)))
    with pytest.raises(ValueError):
        oracle_mod.decode_attention(q, k, k, np.array([1]), 1.0)            # Hq % Hkv
    with pytest.raises(ValueError):
        oracle_mod.decode_attention(f16(np.zeros((1, 2, 8))), k, k, np.array([5]), 1.0)   # len > S_max
