"""Pins for the oracle's statement of the paper's bias rule (Sec. III (i), Eq. (exp bias); Sec. IV-B,
Eq. (approximate)): moment sums, the GenNorm fit by moment matching, the printed polynomial, and the
conversion / averaging with a real multiplier.

The reading itself (bias = multiplier on the gradient, "sigma" = the GenNorm scale parameter) is pinned
by brute force: the L2-optimal multiplier of a 4-bit sign/mantissa/exponent grid, found by numerical
integration against the GenNorm density with a quantiser written here from an explicit level list,
reproduces the printed polynomial to about one per cent over the range the paper plots.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import integrate, optimize, special, stats

import oracle
import co3_inputs as inp


def gennorm_pdf(x, beta, alpha):
    return beta / (2 * alpha * special.gamma(1 / beta)) * np.exp(-(np.abs(x) / alpha) ** beta)


def l2_loss(levels, c, beta, alpha):
    """E (Q(cG)/c - G)^2 for the nearest-level quantiser on `levels` (sorted magnitudes incl. 0)."""
    lv = np.asarray(levels, dtype=np.float64) / c
    th = np.concatenate([[0.0], 0.5 * (lv[1:] + lv[:-1]), [np.inf]])
    tot = 0.0
    for k in range(lv.size):
        v, _ = integrate.quad(lambda x: (x - lv[k]) ** 2 * gennorm_pdf(x, beta, alpha), th[k], th[k + 1], limit=200)
        tot += 2.0 * v
    return tot


def best_multiplier(levels, beta, alpha):
    r = optimize.minimize_scalar(lambda lc: l2_loss(levels, math.exp(lc), beta, alpha),
                                 bounds=(math.log(1e-3 / alpha), math.log(1e2 / alpha)), method="bounded",
                                 options={"xatol": 1e-5})
    return math.exp(r.x)


def printed_poly(beta, golden_dir):
    line = [l for l in open(os.path.join(str(golden_dir), "bias_polynomial.txt")) if not l.startswith("#")][0]
    c = [Fraction(t) for t in line.split()]
    b = Fraction(beta)
    return float(sum(ck * b ** k for k, ck in enumerate(c)))


# ------------------------------------------------------------------ polynomial
def test_polynomial_matches_printed_coefficients(golden_dir):
    for beta in ("0.4", "0.55", "0.8", "1", "1.25", "1.6"):
        assert oracle.bias_poly(float(Fraction(beta))) == pytest.approx(printed_poly(beta, golden_dir), rel=1e-13)
    # clamped outside the plotted range
    assert oracle.bias_poly(0.1) == oracle.bias_poly(0.4)
    assert oracle.bias_poly(7.0) == oracle.bias_poly(1.6)


@pytest.mark.parametrize("beta", [0.8, 1.0, 1.2, 1.4, 1.6])
def test_reading_reproduces_the_printed_fit(beta, golden_dir):
    """fp4 as the paper writes it (sign x mantissa x 2^exponent, 2 mantissa bits, 1 exponent bit, no hidden
    bit): magnitudes {0, .5, 1, 1.5} x {1, 2}.  For GenNorm(beta, alpha = 1) the L2-optimal multiplier equals
    the printed polynomial within 1.5 %; for another alpha it scales as 1/alpha."""
    levels = sorted({m / 2.0 * e for m in range(4) for e in (1, 2)})
    want = printed_poly(str(beta), golden_dir)
    got = best_multiplier(levels, beta, 1.0)
    assert got == pytest.approx(want, rel=0.015)
    alpha = 0.01
    assert best_multiplier(levels, beta, alpha) == pytest.approx(want / alpha, rel=0.015)
    # the rule under test returns exactly that quantity
    assert float(oracle.bias_scale(beta, alpha)) == pytest.approx(want / alpha, rel=1e-6)


@pytest.mark.parametrize("beta,lo,hi", [(0.7, 0.96, 1.0), (0.6, 0.94, 0.98), (0.5, 0.96, 1.0), (0.4, 1.15, 1.3), (0.35, 0.6, 0.8)])
def test_printed_fit_towards_the_low_end_of_the_plotted_range(beta, lo, hi, golden_dir):
    """The figure of Sec. IV-B spans beta from 0.3 to 1.6.  Down to 0.5 the printed quartic stays within 4 % of
    the brute-force optimum (same grid and reading as above); at 0.4 the optimum is 22 % above it, at 0.35
    30 % below it (the quartic has its minimum, 0.006, near 0.36, while the optimum keeps falling towards 0):
    below 0.4 the approximation no longer describes the optimum, which is why the rule limits beta to
    [0.4, 1.6] inside the polynomial."""
    levels = sorted({m / 2.0 * e for m in range(4) for e in (1, 2)})
    ratio = best_multiplier(levels, beta, 1.0) / printed_poly(str(beta), golden_dir)
    assert lo < ratio < hi, ratio
    if beta < 0.4:
        assert oracle.bias_poly(beta) == oracle.bias_poly(0.4)


def test_unit_variance_reading_does_not_fit(golden_dir):
    """With sigma read as the standard deviation the optimum is 2.4 x the polynomial at beta = 0.8: that
    reading is rejected."""
    levels = sorted({m / 2.0 * e for m in range(4) for e in (1, 2)})
    beta = 0.8
    alpha_unit_var = math.sqrt(special.gamma(1 / beta) / special.gamma(3 / beta))
    got = best_multiplier(levels, beta, alpha_unit_var)
    assert got / printed_poly("0.8", golden_dir) > 2.0


def test_own_grid_offset_is_documented_value():
    """On the codec's own 4-bit grid (E1M2 with hidden bit and gradual underflow, anchor 1: 0 .. 3.5 in steps
    of 0.5) the optimum sits 10-15 % above the polynomial and costs under 12 % in squared error: the rule is
    kept as printed."""
    f = oracle.Fmt(1, 2)
    levels = sorted({oracle.level(c >> 2, c & 3, 1, f) for c in range(8)})
    assert levels == [0.5 * k for k in range(8)]
    for beta in (0.8, 1.2, 1.6):
        ratio = best_multiplier(levels, beta, 1.0) / oracle.bias_poly(beta)
        assert 1.05 < ratio < 1.17
        c = oracle.bias_poly(beta)
        assert l2_loss(levels, c, beta, 1.0) < 1.12 * l2_loss(levels, c * ratio, beta, 1.0)


def test_scale_limits():
    assert oracle.bias_scale(1.0, 0.0) == np.float32(1.0)
    assert oracle.bias_scale(1.0, 1e-300) == np.float32(2.0 ** 96)
    assert oracle.bias_scale(1.0, 1e300) == np.float32(2.0 ** -96)


# ------------------------------------------------------------------ moments and fit
def test_ratio_closed_forms():
    assert oracle.gennorm_ratio(2.0) == pytest.approx(2 / math.pi, rel=1e-14)      # Gaussian
    assert oracle.gennorm_ratio(1.0) == pytest.approx(0.5, rel=1e-14)              # Laplace
    assert oracle.gennorm_ratio(400.0) == pytest.approx(0.75, rel=1e-4)            # uniform limit
    b = np.linspace(0.06, 40, 500)
    r = np.array([oracle.gennorm_ratio(x) for x in b])
    assert np.all(np.diff(r) > 0)


@pytest.mark.parametrize("beta", [0.3, 0.5, 0.8, 1.0, 1.37, 2.0, 5.0])
@pytest.mark.parametrize("alpha", [1e-4, 1.0, 30.0])
def test_fit_inverts_population_moments(beta, alpha):
    """Moments by numerical integration of the density (independent of the oracle's gamma formulas)."""
    d = stats.gennorm(beta, scale=alpha)
    upper = d.ppf(1 - 1e-15)
    pts = [alpha * t for t in (1e-3, 1e-1, 1.0, 10.0) if alpha * t < upper]
    m1 = 2 * integrate.quad(lambda x: x * d.pdf(x), 0, upper, points=pts, limit=400, epsabs=0, epsrel=1e-12)[0]
    m2 = 2 * integrate.quad(lambda x: x * x * d.pdf(x), 0, upper, points=pts, limit=400, epsabs=0, epsrel=1e-12)[0]
    n = 1000
    b, a = oracle.gennorm_fit(m1 * n, m2 * n, n)
    assert b == pytest.approx(beta, rel=1e-6)
    assert a == pytest.approx(alpha, rel=1e-6)


def test_fit_on_samples():
    for k, beta in enumerate((0.6, 1.0, 1.5)):
        x = inp.gennorm(inp.rng_for(9, 1, k), 400_000, beta, 2e-3)
        ms = oracle.moments(x, np.zeros_like(x), 1.0)
        b, a = oracle.gennorm_fit(ms[0, 0], ms[0, 1], x.size)
        assert b == pytest.approx(beta, rel=0.03)
        assert a == pytest.approx(2e-3, rel=0.05)


def test_fit_degenerate():
    assert oracle.gennorm_fit(0.0, 0.0, 10) == (1.0, 0.0)
    assert oracle.gennorm_fit(0.0, 0.0, 0) == (1.0, 0.0)
    b, a = oracle.gennorm_fit(10.0, 10.0, 10)          # |x| = 1 everywhere: ratio 1 > 3/4 -> upper end
    assert b == 50.0
    b, a = oracle.gennorm_fit(1.0, 1.0, 10 ** 9)       # a single spike: ratio ~ 0 -> lower end
    assert b == 0.05


def test_moments_against_exact_sums():
    rng = inp.rng_for(9, 2)
    g = inp.gennorm(rng, 50_000, 0.8, 1e-2)
    e = inp.gennorm(rng, 50_000, 1.0, 1e-3)
    seg = [0, 10, 4097, 4097, 50_000]
    for gamma in (1.0, 0.9, 0.0):
        ms = oracle.moments(g, e, gamma, seg)
        x = (g + (np.float32(gamma) * e).astype(np.float32)).astype(np.float32).astype(np.float64)
        for s in range(4):
            xs = x[seg[s]:seg[s + 1]]
            assert ms[s, 0] == pytest.approx(math.fsum(np.abs(xs)), rel=1e-12, abs=0)
            assert ms[s, 1] == pytest.approx(math.fsum(xs * xs), rel=1e-12, abs=0)
    assert np.all(oracle.moments(g, e, 1.0, seg)[2] == 0.0)


# ------------------------------------------------------------------ conversion with a multiplier
@pytest.mark.parametrize("E,M", [(1, 2), (3, 1), (4, 3)])
def test_power_of_two_multiplier_is_an_anchor_shift(E, M):
    """c = 2^k scales exactly: same symbols and same new error as the plain conversion with anchor A - k."""
    f = oracle.Fmt(E, M)
    rng = inp.rng_for(9, 3, E, M)
    g = inp.gennorm(rng, 20_000, 1.0, 1e-3)
    e = inp.gennorm(rng, 20_000, 1.0, 1e-4)
    seg = [0, 777, 20_000]
    A = np.array([3, 5], np.int32)
    for k in (-7, 0, 4, 11):
        c = np.full(2, 2.0 ** k, np.float32)
        s1, e1 = oracle.convert_ef(g, e, A, 0.9, f, seg, scale=c)
        s0, e0 = oracle.convert_ef(g, e, A - k, 0.9, f, seg)
        assert np.array_equal(s1, s0)
        assert np.array_equal(e1.view(np.uint32), e0.view(np.uint32))
        sy = np.stack([s1, s1[::-1].copy()])
        a1 = oracle.aggregate(sy, np.stack([A, A]), f, seg, scale=np.stack([c, c]))
        a0 = oracle.aggregate(sy, np.stack([A - k, A - k]), f, seg)
        assert np.array_equal(a1.view(np.uint32), a0.view(np.uint32))


def test_scaled_conversion_identities():
    """m' = x - fl(level / c) exactly as stated; |c x - level| is within half a quantum unless saturated."""
    f = oracle.Fmt(1, 2)
    rng = inp.rng_for(9, 4)
    g = inp.gennorm(rng, 30_000, 1.0, 1e-3)
    e = inp.gennorm(rng, 30_000, 1.0, 1e-4)
    c = np.array([oracle.bias_scale(1.0, 1e-3)], np.float32)
    A = np.array([1], np.int32)
    sym, e_new = oracle.convert_ef(g, e, A, 1.0, f, scale=c)
    x = (g + e).astype(np.float32)
    y = (c[0] * x).astype(np.float32)
    val = np.array([oracle.symbol_value(int(q), 1, f) for q in range(f.K)], np.float32)[sym]
    ghat = (val / c[0]).astype(np.float32)
    assert np.array_equal(e_new.view(np.uint32), (x - ghat).astype(np.float32).view(np.uint32))
    inside = np.abs(y) <= 3.5
    assert np.all(np.abs(y[inside].astype(np.float64) - val[inside]) <= 0.25)
    assert np.all(np.abs(val[~inside]) == 3.5)
    # scalar agreement with the value-level quantiser
    want = oracle.quantize_values(y, 1, 1, 2)
    assert np.array_equal(want, val.astype(np.float64))


def test_aggregate_scaled_against_float64():
    f = oracle.Fmt(3, 1)
    rng = inp.rng_for(9, 5)
    U, n = 5, 4000
    sym = rng.integers(0, f.K, size=(U, n)).astype(np.uint8)
    A = rng.integers(-3, 3, size=(U, 1)).astype(np.int32)
    c = rng.uniform(0.3, 900.0, size=(U, 1)).astype(np.float32)
    got = oracle.aggregate(sym, A, f, scale=c)
    ref = np.zeros(n)
    mag = np.zeros(n)
    for u in range(U):
        v = np.array([oracle.symbol_value(q, int(A[u, 0]), f) for q in range(f.K)], np.float64)[sym[u]]
        ref += v / float(c[u, 0])
        mag += np.abs(v) / float(c[u, 0])
    assert np.all(np.abs(got - ref / U) <= 1e-6 * mag / U + 1e-45)


def test_rule_beats_max_anchor_in_l2():
    """What the bias is for (Sec. III (i)): smaller expected squared error than anchoring the grid to the
    largest magnitude, on the 4-bit format, for GenNorm gradients."""
    f = oracle.Fmt(1, 2)
    for k, beta in enumerate((0.8, 1.0, 1.5)):
        g = inp.gennorm(inp.rng_for(9, 6, k), 200_000, beta, 1e-3)
        z = np.zeros_like(g)
        c = oracle.bias_scales(g, z, 1.0)
        _, e_rule = oracle.convert_ef(g, z, np.array([1], np.int32), 1.0, f, scale=c)
        _, e_max = oracle.convert_ef(g, z, oracle.anchor(g, f), 1.0, f)
        assert np.sum(e_rule.astype(np.float64) ** 2) < 0.5 * np.sum(e_max.astype(np.float64) ** 2)
