"""Pins for the fp64 oracle: every expected value here comes from a closed form,
exact rational arithmetic, an independent library routine or the paper's printed
numbers -- never from the oracle itself or from the HIP path."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

from paper_2605_25655_amd import synth


def f16(a):
    return np.asarray(a, dtype=np.float16)


def frac_of_half(v) -> Fraction:
    """Exact rational value of an fp16 number, decoded from its bit pattern."""
    bits = int(np.asarray(v, np.float16).view(np.uint16))
    sign = -1 if bits >> 15 else 1
    e = (bits >> 10) & 0x1F
    m = bits & 0x3FF
    assert e != 31
    if e == 0:
        return sign * Fraction(m, 1 << 24)
    return sign * Fraction(1024 + m, 1024) * (Fraction(2) ** (e - 15))


# ---------------------------------------------------------------- fp16 decode
def test_half_decode_every_finite_pattern(oracle_mod):
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)       # numpy's own widening
    for b in list(range(0, 1 << 16, 97)) + [0x0001, 0x03FF, 0x0400, 0x7BFF, 0x8001, 0xFBFF, 0x3C00]:
        got = oracle_mod.half_to_double(b)
        exp = ref[b]
        if np.isnan(exp):
            assert np.isnan(got)
        else:
            assert got == exp, hex(b)
    assert oracle_mod.half_to_double(0x0001) == 2.0 ** -24
    assert oracle_mod.half_to_double(0x7BFF) == 65504.0
    assert oracle_mod.half_to_double(0x7C00) == float("inf")
    assert np.signbit(oracle_mod.half_to_double(0x8000))


# -------------------------------------------------------------------- linear
def test_identity_weights_return_x_exactly(oracle_mod):
    K = 64
    x = f16(np.random.default_rng(1).standard_normal((3, K)))
    x[0, 0] = np.float16(6.0e-8)      # subnormal
    x[1, 5] = np.float16(65504.0)     # max finite
    x[2, 7] = np.float16(-6.1e-5)     # smallest normal-ish
    y, s = oracle_mod.linear(x, f16(np.eye(K)))
    assert np.array_equal(y, x.astype(np.float64))
    assert np.array_equal(s, np.abs(x.astype(np.float64)))


def test_one_hot_rows_gather(oracle_mod):
    rng = np.random.default_rng(2)
    M, N, K = 4, 37, 48
    perm = rng.integers(0, K, size=N)
    w = np.zeros((N, K), np.float16)
    w[np.arange(N), perm] = 1
    x = f16(rng.standard_normal((M, K)))
    y, s = oracle_mod.linear(x, w)
    assert np.array_equal(y, x.astype(np.float64)[:, perm])
    assert np.array_equal(s, np.abs(y))


def test_transposed_operand_would_fail(oracle_mod):
    """w is [N,K]: a one-hot at (n=1,k=2) must route x[:,2] to output 1, not x[:,1] to 2."""
    w = np.zeros((3, 3), np.float16)
    w[1, 2] = 1
    x = f16([[10, 20, 30]])
    y, _ = oracle_mod.linear(x, w)
    assert y.tolist() == [[0.0, 30.0, 0.0]]


def test_all_ones_weights_constant_x(oracle_mod):
    K = 4096
    x = np.full((2, K), 2.0 ** -6, np.float16)
    y, s = oracle_mod.linear(x, np.ones((5, K), np.float16))
    assert np.all(y == 64.0) and np.all(s == 64.0)


def test_signed_unit_weights_count(oracle_mod):
    rng = np.random.default_rng(3)
    K, N = 1000, 9
    sign = rng.choice([-1.0, 1.0], size=(N, K))
    y, s = oracle_mod.linear(np.ones((1, K), np.float16), f16(sign))
    assert np.array_equal(y[0], (sign > 0).sum(1) - (sign < 0).sum(1))
    assert np.all(s == K)


def test_linearity(oracle_mod):
    rng = np.random.default_rng(4)
    x1 = f16(rng.integers(-8, 8, size=(3, 40)))
    x2 = f16(rng.integers(-8, 8, size=(3, 40)))
    w = f16(rng.standard_normal((11, 40)) * 0.02)
    ya, _ = oracle_mod.linear(x1, w)
    yb, _ = oracle_mod.linear(x2, w)
    yc, _ = oracle_mod.linear(f16(x1.astype(np.float64) + x2.astype(np.float64)), w)
    np.testing.assert_allclose(yc, ya + yb, rtol=0, atol=1e-13)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 4), (4, 4, 8), (3, 2, 5), (1, 4, 3)])
def test_brute_force_rational_linear(oracle_mod, M, N, K):
    rng = np.random.default_rng(100 + M * 16 + N * 4 + K)
    x = f16(rng.integers(-12, 13, size=(M, K)) / 8.0)
    w = f16(rng.integers(-12, 13, size=(N, K)) / 64.0)
    y, s = oracle_mod.linear(x, w)
    for m in range(M):
        for n in range(N):
            terms = [frac_of_half(x[m, k]) * frac_of_half(w[n, k]) for k in range(K)]
            assert Fraction(y[m, n]) == sum(terms)
            assert Fraction(s[m, n]) == sum(abs(t) for t in terms)


def test_numpy_fp64_witness_mid_size(oracle_mod):
    x, w, _ = synth.random_problem(77, 5, 300, 1376)
    y, s = oracle_mod.linear(x, w)
    xd, wd = x.astype(np.float64), w.astype(np.float64)
    ref = xd @ wd.T
    sref = np.abs(xd) @ np.abs(wd).T
    assert np.max(np.abs(y - ref) / sref) < 1e-12
    assert np.max(np.abs(s - sref) / sref) < 1e-12


# ------------------------------------------------------------------- rmsnorm
def test_rmsnorm_constant_vector_closed_form(oracle_mod):
    K = 256
    for c in (1.0, -1.0, 0.5, 3.0):
        x = np.full((1, K), c, np.float16)
        y, s = oracle_mod.rmsnorm_qkv(x, np.ones(K, np.float16), 1e-6, f16(np.eye(K)))
        eps = float(np.float32(1e-6))
        exp = c / np.sqrt(c * c + eps)
        np.testing.assert_allclose(y, exp, rtol=2e-16 * 8)
        np.testing.assert_allclose(s, abs(exp), rtol=2e-16 * 8)
    # the c = 1 value to 15 digits: 1/sqrt(1 + 1e-6f)
    x = np.ones((1, K), np.float16)
    y, _ = oracle_mod.rmsnorm_qkv(x, np.ones(K, np.float16), 1e-6, f16(np.eye(K)))
    assert abs(y[0, 0] - 0.999999500000375) < 2e-14


def test_rmsnorm_signs_have_same_scale(oracle_mod):
    rng = np.random.default_rng(5)
    K = 128
    sgn = rng.choice([-1.0, 1.0], size=(1, K))
    y, _ = oracle_mod.rmsnorm_qkv(f16(sgn), np.ones(K, np.float16), 1e-6, f16(np.eye(K)))
    r = 1 / np.sqrt(1 + float(np.float32(1e-6)))
    np.testing.assert_allclose(y, sgn * r, rtol=1e-15)


def test_rmsnorm_scale_invariance_eps0(oracle_mod):
    x, w, g = synth.random_problem(6, 3, 20, 64)
    y1, _ = oracle_mod.rmsnorm_qkv(x, g, 0.0, w)
    y2, _ = oracle_mod.rmsnorm_qkv(f16(x.astype(np.float64) * 4), g, 0.0, w)
    np.testing.assert_allclose(y2, y1, rtol=1e-13, atol=1e-15)


def test_rmsnorm_uses_gamma_not_one_plus_gamma_and_no_mean_subtraction(oracle_mod):
    K = 8
    x = f16([[1, 2, 3, 4, 5, 6, 7, 8]])
    g = f16([2, 2, 2, 2, 0.5, 0.5, 0.5, 0.5])
    y, _ = oracle_mod.rmsnorm_qkv(x, g, 0.0, f16(np.eye(K)))
    ms = Fraction(sum(i * i for i in range(1, 9)), 8)          # 25.5, no mean removed
    exp = np.array([i * float(gv) for i, gv in zip(range(1, 9), g)]) / np.sqrt(float(ms))
    np.testing.assert_allclose(y[0], exp, rtol=1e-15)


def test_rmsnorm_factorisation_against_linear(oracle_mod):
    """rmsnorm(x) W^T == r_m * ((x*gamma) W^T): checked with an independent numpy
    fp64 evaluation of the right-hand side."""
    x, w, g = synth.random_problem(8, 4, 50, 96)
    eps = 1e-6
    y, s = oracle_mod.rmsnorm_qkv(x, g, eps, w)
    xd, gd, wd = x.astype(np.float64), g.astype(np.float64), w.astype(np.float64)
    r = 1 / np.sqrt((xd ** 2).mean(1, keepdims=True) + float(np.float32(eps)))
    ref = r * ((xd * gd) @ wd.T)
    sref = r * (np.abs(xd * gd) @ np.abs(wd).T)
    assert np.max(np.abs(y - ref) / sref) < 1e-13
    assert np.max(np.abs(s - sref) / sref) < 1e-13


def test_rmsnorm_eps_is_the_fp32_value(oracle_mod):
    """With x == 0 the only term under the root is eps; 1e-6f != 1e-6."""
    K = 16
    x = np.zeros((1, K), np.float16)
    x[0, 0] = np.float16(2.0 ** -14)
    y, _ = oracle_mod.rmsnorm_qkv(x, np.ones(K, np.float16), 1e-6, f16(np.eye(K)))
    eps32 = Fraction(float(np.float32(1e-6)))
    ms = Fraction(1, 2 ** 28) / K
    exp = float(Fraction(1, 2 ** 14)) / np.sqrt(float(ms + eps32))
    assert abs(y[0, 0] - exp) <= 4e-16 * abs(exp)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 2, 3), (3, 4, 8)])
def test_brute_force_rational_rmsnorm(oracle_mod, M, N, K):
    rng = np.random.default_rng(200 + M + N + K)
    x = f16(rng.integers(-9, 10, size=(M, K)) / 4.0)
    x[:, 0] = 1
    g = f16(1 + rng.integers(-3, 4, size=K) / 16.0)
    w = f16(rng.integers(-9, 10, size=(N, K)) / 32.0)
    eps = 2.0 ** -10
    y, s = oracle_mod.rmsnorm_qkv(x, g, eps, w)
    getcontext().prec = 60
    for m in range(M):
        ms = sum(frac_of_half(x[m, k]) ** 2 for k in range(K)) / K + Fraction(eps)
        r = 1 / (Decimal(ms.numerator) / Decimal(ms.denominator)).sqrt()
        for n in range(N):
            t = [frac_of_half(x[m, k]) * frac_of_half(g[k]) * frac_of_half(w[n, k]) for k in range(K)]
            tot, mag = sum(t), sum(abs(v) for v in t)
            exp = float(Decimal(tot.numerator) / Decimal(tot.denominator) * r)
            exps = float(Decimal(mag.numerator) / Decimal(mag.denominator) * r)
            assert abs(y[m, n] - exp) <= 1e-15 * max(exps, 1e-300)
            assert abs(s[m, n] - exps) <= 1e-15 * max(exps, 1e-300)


# ---------------------------------------------------------------------- silu
def test_silu_reference_values(oracle_mod):
    getcontext().prec = 50
    for t in ("0", "1", "-1", "2", "-2", "8", "-20", "0.5", "-1.2784645427610738", "30", "-30"):
        d = Decimal(t)
        exp = float(d / (1 + (-d).exp()))
        got = oracle_mod.silu(float(t))
        assert abs(got - exp) <= 4e-16 * abs(exp), t
    assert oracle_mod.silu(0.0) == 0.0
    assert abs(oracle_mod.silu(1.0) - 0.7310585786300049) < 1e-15       # = sigmoid(1)
    assert abs(oracle_mod.silu(-1.0) + 0.2689414213699951) < 1e-15


def test_silu_identities(oracle_mod):
    for t in np.linspace(-12, 12, 49):
        assert abs(oracle_mod.silu(t) - oracle_mod.silu(-t) - t) < 1e-14
    ts = np.linspace(-3, 0, 3001)
    vals = np.array([oracle_mod.silu(t) for t in ts])
    i = int(np.argmin(vals))
    assert abs(ts[i] - (-1.2784645427610738)) < 2e-3
    assert abs(vals[i] - (-0.27846454276107374)) < 1e-6


# -------------------------------------------------------------------- swiglu
def test_swiglu_selector_matrices_closed_form(oracle_mod):
    rng = np.random.default_rng(9)
    M, H, I = 3, 16, 24
    x = f16(rng.standard_normal((M, H)))
    p, q = rng.integers(0, H, I), rng.integers(0, H, I)
    wg = np.zeros((I, H), np.float16); wg[np.arange(I), p] = 1
    wu = np.zeros((I, H), np.float16); wu[np.arange(I), q] = 1
    d = rng.integers(0, I, H)
    wd = np.zeros((H, I), np.float16); wd[np.arange(H), d] = 1
    y, s, h = oracle_mod.swiglu_mlp(x, wg, wu, wd, return_h=True)
    xd = x.astype(np.float64)
    getcontext().prec = 40
    for m in range(M):
        for n in range(H):
            g, u = xd[m, p[d[n]]], xd[m, q[d[n]]]
            exp = float(Decimal(g) / (1 + (-Decimal(g)).exp()) * Decimal(u))
            assert abs(y[m, n] - exp) <= 1e-15 * max(abs(exp), 1e-300)
            assert abs(s[m, n] - abs(exp)) <= 1e-15 * max(abs(exp), 1e-300)


def test_swiglu_gate_and_up_are_not_swapped(oracle_mod):
    H, I = 2, 1
    x = f16([[2.0, -3.0]])
    wg = f16([[1, 0]]); wu = f16([[0, 1]]); wd = f16([[1], [0]])
    y, _ = oracle_mod.swiglu_mlp(x, wg, wu, wd)
    silu2 = 2 / (1 + np.exp(-2.0))
    assert abs(y[0, 0] - silu2 * -3.0) < 1e-15        # silu(gate) * up
    assert y[0, 1] == 0.0


def test_gate_up_alone_matches_the_mlp_oracle_and_its_magnitude_is_first_order(oracle_mod):
    """h from swiglu_gate_up is the h the (pinned) MLP oracle forms; S_h is pinned three ways: the closed form
    for selector weights, the derivative silu' against a central difference of the C silu, and the defining
    property -- moving g by eps*S_g and u by eps*S_u (worst signs) moves h by eps*S_h to first order."""
    rng = np.random.default_rng(21)
    M, H, I = 4, 32, 40
    x = f16(rng.standard_normal((M, H)))
    wg, wu = f16(rng.standard_normal((I, H)) * 0.3), f16(rng.standard_normal((I, H)) * 0.3)
    h, sh = oracle_mod.swiglu_gate_up(x, wg, wu)
    _, _, h_mlp = oracle_mod.swiglu_mlp(x, wg, wu, np.zeros((H, I), np.float16), return_h=True)
    np.testing.assert_allclose(h, h_mlp, rtol=1e-14, atol=1e-300)
    g, sg = oracle_mod.linear(x, wg)
    u, su = oracle_mod.linear(x, wu)
    eps = 1e-7
    silu = np.vectorize(oracle_mod.silu)
    worst = np.zeros_like(h)
    for dg in (-1, 1):
        for du in (-1, 1):
            hp = silu(g + dg * eps * sg) * (u + du * eps * su)
            worst = np.maximum(worst, np.abs(hp - h))
    np.testing.assert_allclose(worst, eps * sh, rtol=1e-4, atol=1e-18)
    # selector weights: g = x[p], u = x[q], S_g = |x[p]|, S_u = |x[q]|
    p_, q_ = rng.integers(0, H, I), rng.integers(0, H, I)
    sel_g = np.zeros((I, H), np.float16); sel_g[np.arange(I), p_] = 1
    sel_u = np.zeros((I, H), np.float16); sel_u[np.arange(I), q_] = 1
    h2, s2 = oracle_mod.swiglu_gate_up(x, sel_g, sel_u)
    xd = x.astype(np.float64)
    gg, uu = xd[:, p_], xd[:, q_]
    d = 1e-6
    dsilu = (silu(gg + d) - silu(gg - d)) / (2 * d)
    np.testing.assert_allclose(h2, silu(gg) * uu, rtol=1e-15)
    np.testing.assert_allclose(s2, np.abs(dsilu * uu) * np.abs(gg) + np.abs(silu(gg)) * np.abs(uu), rtol=1e-8, atol=1e-12)


def test_swiglu_composition_with_numpy_witness(oracle_mod):
    cfg = synth.CONFIGS[1]
    rng = np.random.Generator(np.random.Philox(key=11))
    M, H, I = 2, 64, 88
    x = f16(rng.standard_normal((M, H)))
    wg, wu = f16(rng.standard_normal((I, H)) * 0.2), f16(rng.standard_normal((I, H)) * 0.2)
    wd = f16(rng.standard_normal((H, I)) * cfg.sigma_w)
    y, s, h = oracle_mod.swiglu_mlp(x, wg, wu, wd, return_h=True)
    xd = x.astype(np.float64)
    g, u = xd @ wg.astype(np.float64).T, xd @ wu.astype(np.float64).T
    href = g / (1 + np.exp(-g)) * u
    yref = href @ wd.astype(np.float64).T
    sref = np.abs(href) @ np.abs(wd.astype(np.float64)).T
    np.testing.assert_allclose(h, href, rtol=1e-13, atol=1e-16)
    assert np.max(np.abs(y - yref) / sref) < 1e-12
    assert np.max(np.abs(s - sref) / sref) < 1e-12
    # and the pieces agree with two oracle linear calls (same values, no rounding in between)
    g2, _ = oracle_mod.linear(x, wg)
    np.testing.assert_allclose(g2, g, rtol=1e-13, atol=1e-16)


# ------------------------------------------------------- tolerance has teeth
def test_acceptance_rule_has_teeth(oracle_mod):
    """Plausible kernel mistakes must fail the rule: a dropped ragged tail, one
    corrupted weight, fp16 (instead of fp32) accumulation of same-sign terms, a
    swapped argmax."""
    from tests.parity import check
    x, w, _ = synth.random_problem(13, 2, 64, 512)
    y, s = oracle_mod.linear(x, w)
    good = y.astype(np.float16)                       # correctly rounded result passes
    check(good, y, s, "rounded")
    xd, wd = x.astype(np.float64), w.astype(np.float64)
    tail = (xd[:, :480] @ wd[:, :480].T).astype(np.float16)      # last 32 terms dropped
    with pytest.raises(AssertionError):
        check(tail, y, s, "dropped-tail", argmax=False)
    w2 = w.copy()
    big = int(np.argmax(np.abs(x[0])))
    w2[7, big] = np.float16(float(w2[7, big]) + 0.25)   # one corrupted weight
    ybad = (xd @ w2.astype(np.float64).T).astype(np.float16)
    with pytest.raises(AssertionError):
        check(ybad, y, s, "perturbed", argmax=False)
    swapped = good.copy()                              # argmax rule has teeth too
    t = int(np.argmax(y[0])); o = (t + 1) % 64
    swapped[0, [t, o]] = swapped[0, [o, t]]
    with pytest.raises(AssertionError):
        check(swapped, y, s, "argmax")
    # fp16 running sum of 8192 positive terms stalls once the sum's ulp exceeds the terms
    K = 8192
    xp = np.full((1, K), 1.0, np.float16)
    wp = np.full((4, K), 0.25, np.float16)
    yp, sp = oracle_mod.linear(xp, wp)
    acc = np.zeros((1, 4), np.float16)
    for k in range(K):
        acc = (acc + xp[:, k:k + 1] * wp[:, k][None, :]).astype(np.float16)
    with pytest.raises(AssertionError):
        check(acc, yp, sp, "fp16-accumulate", argmax=False)


def test_thread_count_does_not_change_results(oracle_mod):
    x, w, g = synth.random_problem(14, 3, 129, 200)
    y1, s1 = oracle_mod.rmsnorm_qkv(x, g, 1e-6, w)
    y2, s2 = oracle_mod.rmsnorm_qkv(x, g, 1e-6, w)
    assert np.array_equal(y1, y2) and np.array_equal(s1, s2)
