"""Pins for the oracle's layer-closing operators (residual additions, RMSNorm in front of the MLP).

Each check fixes the oracle against something other than itself: exact integer arithmetic, exact
rational brute force, closed forms, or its own separately pinned parts composed by hand."""
from fractions import Fraction

import numpy as np
import pytest


def f16(a):
    return np.asarray(a, dtype=np.float16)


def frac(v) -> Fraction:
    return Fraction(float(v))


def test_residual_cancels_an_integer_product_exactly(oracle_mod):
    # small integers: every product and sum is exact in fp16, so res = -(x w^T) gives exactly zero
    rng = np.random.default_rng(5)
    x = f16(rng.integers(-3, 4, size=(4, 16)))
    w = f16(rng.integers(-2, 3, size=(6, 16)))
    prod = x.astype(np.int64) @ w.astype(np.int64).T
    y, s = oracle_mod.linear_residual(x, w, f16(-prod))
    assert np.array_equal(y, np.zeros_like(y))
    assert np.array_equal(s, np.abs(x.astype(np.int64))[:, None, :].__mul__(np.abs(w.astype(np.int64))[None]).sum(-1)
                          + np.abs(prod))


def test_residual_is_added_not_subtracted_and_not_transposed(oracle_mod):
    x = f16(np.zeros((2, 8)))
    w = f16(np.ones((3, 8)))
    res = f16([[1, 2, 3], [-4, 5, -6]])
    y, s = oracle_mod.linear_residual(x, w, res)
    assert np.array_equal(y, res.astype(np.float64))
    assert np.array_equal(s, np.abs(res.astype(np.float64)))


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 4), (3, 2, 5)])
def test_brute_force_rational_linear_residual(oracle_mod, M, N, K):
    rng = np.random.default_rng(100 + M + N + K)
    x, w, r = f16(rng.standard_normal((M, K))), f16(rng.standard_normal((N, K))), f16(rng.standard_normal((M, N)))
    y, s = oracle_mod.linear_residual(x, w, r)
    for m in range(M):
        for n in range(N):
            exact = frac(r[m, n]) + sum(frac(x[m, k]) * frac(w[n, k]) for k in range(K))
            mag = abs(frac(r[m, n])) + sum(abs(frac(x[m, k]) * frac(w[n, k])) for k in range(K))
            assert abs(Fraction(y[m, n]) - exact) <= Fraction(1, 2 ** 45) * max(mag, Fraction(1, 2 ** 30))
            assert abs(Fraction(s[m, n]) - mag) <= Fraction(1, 2 ** 45) * max(mag, Fraction(1, 2 ** 30))


def test_normalised_mlp_is_the_pinned_parts_composed(oracle_mod):
    # n = rmsnorm(x) formed here in fp64 from the definition; gate/up/down through the plain-linear oracle
    # (pinned by rational brute force) cannot be used on an fp64 n, so the composition is done with numpy on
    # the exactly widened fp16 values -- a witness that shares nothing with the C loops.
    rng = np.random.default_rng(11)
    M, H, I = 3, 24, 40
    x = f16(rng.standard_normal((M, H)))
    g = f16(1 + 0.1 * rng.standard_normal(H))
    wg, wu = f16(rng.standard_normal((I, H)) * 0.2), f16(rng.standard_normal((I, H)) * 0.2)
    wd = f16(rng.standard_normal((H, I)) * 0.2)
    res = f16(rng.standard_normal((M, H)))
    eps = np.float32(1e-6)
    xd = x.astype(np.float64)
    n = xd / np.sqrt((xd ** 2).mean(1, keepdims=True) + np.float64(eps)) * g.astype(np.float64)
    gate, up = n @ wg.astype(np.float64).T, n @ wu.astype(np.float64).T
    h = gate / (1 + np.exp(-gate)) * up
    want = h @ wd.astype(np.float64).T
    y, s, hh = oracle_mod.rmsnorm_swiglu_mlp(x, g, float(eps), wg, wu, wd, return_h=True)
    np.testing.assert_allclose(hh, h, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(s, np.abs(h)[:, None, :].__mul__(np.abs(wd.astype(np.float64))[None]).sum(-1), rtol=1e-12)
    y2, s2 = oracle_mod.rmsnorm_swiglu_mlp(x, g, float(eps), wg, wu, wd, res=res)
    np.testing.assert_allclose(y2, want + res.astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(s2 - s, np.abs(res.astype(np.float64)), rtol=1e-12, atol=1e-13)


def test_normalised_mlp_constant_rows_closed_form(oracle_mod):
    # x = c everywhere, gamma = 1: n = c / sqrt(c^2 + eps) for every element.  Gate and up select element j
    # (one-hot rows), down is the identity on the first H of I = H columns: y = silu(n) * n.
    H = 16
    c = 3.0
    eps = np.float32(1e-6)
    x = f16(np.full((2, H), c))
    x[1] = -c
    eye = f16(np.eye(H))
    y, s = oracle_mod.rmsnorm_swiglu_mlp(x, f16(np.ones(H)), float(eps), eye, eye, eye)
    n = c / np.sqrt(c * c + np.float64(eps))
    for sign, row in ((1.0, 0), (-1.0, 1)):
        v = sign * n
        want = v / (1 + np.exp(-v)) * v
        np.testing.assert_allclose(y[row], np.full(H, want), rtol=1e-14)
        np.testing.assert_allclose(s[row], np.full(H, abs(want)), rtol=1e-14)


def test_normalised_mlp_agrees_with_the_unnormalised_one_on_prenormalised_input(oracle_mod):
    # rows of +-1 have mean square exactly 1: with eps = 0 and gamma = 1, rmsnorm is the identity
    rng = np.random.default_rng(3)
    M, H, I = 4, 32, 24
    x = f16(rng.choice([-1.0, 1.0], size=(M, H)))
    wg, wu = f16(rng.standard_normal((I, H)) * 0.1), f16(rng.standard_normal((I, H)) * 0.1)
    wd = f16(rng.standard_normal((H, I)) * 0.1)
    y0, s0 = oracle_mod.swiglu_mlp(x, wg, wu, wd)
    y1, s1 = oracle_mod.rmsnorm_swiglu_mlp(x, f16(np.ones(H)), 0.0, wg, wu, wd)
    assert np.array_equal(y0, y1) and np.array_equal(s0, s1)


def test_gamma_scales_the_normalised_input_of_the_mlp(oracle_mod):
    # doubling gamma doubles n, hence gate and up: checked against the unnormalised oracle fed 2x
    rng = np.random.default_rng(8)
    M, H, I = 2, 16, 8
    x = f16(rng.choice([-1.0, 1.0], size=(M, H)))
    wg, wu = f16(rng.standard_normal((I, H)) * 0.1), f16(rng.standard_normal((I, H)) * 0.1)
    wd = f16(rng.standard_normal((H, I)) * 0.1)
    y_ref, _ = oracle_mod.swiglu_mlp(f16(2 * x.astype(np.float32)), wg, wu, wd)
    y, _ = oracle_mod.rmsnorm_swiglu_mlp(x, f16(np.full(H, 2.0)), 0.0, wg, wu, wd)
    assert np.array_equal(y, y_ref)
