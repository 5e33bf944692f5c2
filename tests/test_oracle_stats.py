"""Pins of the oracle's GG statistics (Eq. 1-3, Eq. 5) against closed forms, numerical
integration of the density of Eq. 1, and independent samplers (scipy.stats.gennorm, numpy gamma).
None of the expected values below comes from the oracle or the HIP library."""
import math

import numpy as np
import pytest
from scipy import integrate, stats

import gg_inputs
import oracle


# ---- density of Eq. 1 written out for numerical integration (mu = 0) -------------------------
def ggd_pdf(x, alpha, beta):
    return beta / (2.0 * alpha * math.gamma(1.0 / beta)) * math.exp(-((abs(x) / alpha) ** beta))


def quad_moment(p, alpha, beta):
    # integrate |x|^p f(x) over the real line; substitute x = alpha * t^(1/beta) to tame small beta
    f = lambda t: (alpha * t ** (1.0 / beta)) ** p * math.exp(-t) * t ** (1.0 / beta - 1.0) / math.gamma(1.0 / beta)
    v, _ = integrate.quad(f, 0.0, np.inf, epsabs=0, epsrel=1e-11, limit=400)
    return v


def test_rho_closed_forms():
    assert oracle.rho(1.0) == pytest.approx(0.5, rel=1e-13)            # Laplace: (E|x|)^2/E x^2 = a^2/(2a^2)
    assert oracle.rho(2.0) == pytest.approx(2.0 / math.pi, rel=1e-13)  # Gaussian
    assert oracle.rho(0.5) == pytest.approx(0.3, rel=1e-13)            # Gamma(4)^2/(Gamma(2)Gamma(6)) = 36/120
    assert oracle.rho(1.0 / 3.0) == pytest.approx(math.factorial(5) ** 2 / (2.0 * math.factorial(8)), rel=1e-13)
    assert oracle.rho(1e6) == pytest.approx(0.75, rel=1e-6)            # uniform limit: (1/2)^2/(1/3)


def test_rho_monotone_and_bounded():
    bs = np.geomspace(0.05, 20.0, 400)
    r = np.array([oracle.rho(b) for b in bs])
    assert np.all(np.diff(r) > 0)
    assert r[0] > 0 and r[-1] < 0.75


@pytest.mark.parametrize("beta", [0.3, 0.5, 0.8, 1.0, 1.5, 2.0, 4.0, 10.0])
def test_rho_matches_integrated_density(beta):
    alpha = 0.37
    m1 = quad_moment(1, alpha, beta)
    m2 = quad_moment(2, alpha, beta)
    assert oracle.rho(beta) == pytest.approx(m1 * m1 / m2, rel=1e-8)


def test_density_normalises_and_variance_eq3():
    # sanity of the test's own density, and Eq. 3: D[x] = alpha^2 Gamma(3/b)/Gamma(1/b)
    alpha, beta = 0.02, 1.3
    total, _ = integrate.quad(lambda x: ggd_pdf(x, alpha, beta), -1.0, 1.0, epsabs=0, epsrel=1e-11, points=[0.0])
    assert total == pytest.approx(1.0, rel=1e-9)
    var, _ = integrate.quad(lambda x: x * x * ggd_pdf(x, alpha, beta), -1.0, 1.0, epsabs=0, epsrel=1e-11,
                            points=[0.0])
    # oracle: alpha recovered from the variance via Eq. 2 must be the alpha we started from
    assert oracle.alpha_from_m2(var, beta) == pytest.approx(alpha, rel=1e-8)


@pytest.mark.parametrize("beta,m1_over_a,m2_over_a2", [(1.0, 1.0, 2.0), (2.0, 1.0 / math.sqrt(math.pi), 0.5),
                                                       (0.5, 6.0, 120.0)])
def test_fit_from_exact_moments(beta, m1_over_a, m2_over_a2):
    alpha, n = 0.015, 1_000_000
    f = oracle.fit_from_moments(n * alpha * m1_over_a, n * alpha * alpha * m2_over_a2, n)
    assert f.flags == 0
    assert f.beta == pytest.approx(beta, rel=1e-9)
    assert f.alpha == pytest.approx(alpha, rel=1e-9)


@pytest.mark.parametrize("beta", [0.07, 0.1, 0.33, 0.8, 1.5, 3.0, 7.5, 19.0])
def test_solve_inverts_integrated_rho(beta):
    m1 = quad_moment(1, 1.0, beta)
    m2 = quad_moment(2, 1.0, beta)
    b, fl = oracle.solve_beta(m1 * m1 / m2)
    assert fl == 0
    assert b == pytest.approx(beta, rel=2e-7)


def test_solve_clamps():
    b, fl = oracle.solve_beta(1e-12)
    assert b == oracle.BETA_MIN and fl == oracle.BETA_CLAMPED_LO
    b, fl = oracle.solve_beta(0.7499999)
    assert b == oracle.BETA_MAX and fl == oracle.BETA_CLAMPED_HI
    # a two-valued +-c tensor has rho = 1 > 3/4
    f = oracle.fit(np.array([0.5, -0.5, 0.5, -0.5], dtype=np.float32))
    assert f.flags == oracle.BETA_CLAMPED_HI and f.beta == oracle.BETA_MAX


def test_fit_degenerate_empty_nonfinite():
    f = oracle.fit(np.zeros(0, dtype=np.float32))
    assert f.flags == oracle.EMPTY and f.n == 0 and f.alpha == 0 and f.beta == 0
    f = oracle.fit(np.zeros(100, dtype=np.float32))
    assert f.flags == oracle.DEGENERATE and f.alpha == 0 and f.beta == 2
    f = oracle.fit(np.array([1.0, np.nan, 2.0], dtype=np.float32))
    assert f.flags == oracle.NONFINITE and f.alpha == 0 and f.beta == 2
    f = oracle.fit(np.array([1.0, np.inf], dtype=np.float32))
    assert f.flags == oracle.NONFINITE


def test_moments_small_by_hand():
    x = np.array([1.5, -2.0, 0.0, 0.25, -0.5], dtype=np.float32)
    s1, s2 = oracle.moments(x)
    assert s1 == 4.25 and s2 == 2.25 + 4.0 + 0.0625 + 0.25
    # bf16 inputs are widened exactly: 1.5, -2, 0.25 are bf16-representable
    xb = gg_inputs.f32_to_bf16_bits(np.array([1.5, -2.0, 0.25], dtype=np.float32))
    s1, s2 = oracle.moments(xb)
    assert s1 == 3.75 and s2 == 2.25 + 4.0 + 0.0625


@pytest.mark.parametrize("alpha,beta,seed", [(0.02, 1.0, 0), (0.015, 1.5, 1), (0.5, 0.8, 2), (1e-4, 0.5, 3),
                                             (0.01, 2.0, 4)])
def test_fit_recovers_gennorm_samples(alpha, beta, seed):
    """scipy's generalized normal is exactly Eq. 1; the moment estimator must recover its parameters."""
    n = 4_000_000
    x = stats.gennorm.rvs(beta, scale=alpha, size=n, random_state=np.random.default_rng(seed)).astype(np.float32)
    f = oracle.fit(x)
    assert f.flags == 0 and f.n == n
    assert abs(f.beta - beta) < 0.02
    assert f.alpha == pytest.approx(alpha, rel=0.02 if beta < 0.7 else 0.01)
    # sums against numpy's pairwise double sums
    xd = x.astype(np.float64)
    assert f.sum_abs == pytest.approx(np.abs(xd).sum(), rel=1e-12)
    assert f.sum_sq == pytest.approx((xd * xd).sum(), rel=1e-12)


def test_fit_recovers_numpy_gamma_samples_bf16():
    x = gg_inputs.gg_numpy(2_000_000, 0.015, 1.5, seed=11)
    xb = gg_inputs.f32_to_bf16_bits(x)
    f = oracle.fit(xb)
    assert abs(f.beta - 1.5) < 0.02 and f.alpha == pytest.approx(0.015, rel=0.01)
    # and it equals the fit of the widened values
    f2 = oracle.fit(gg_inputs.bf16_bits_to_f32(xb))
    assert (f.sum_abs, f.sum_sq, f.beta, f.alpha) == (f2.sum_abs, f2.sum_sq, f2.beta, f2.alpha)


def test_fit_is_scale_equivariant():
    x = gg_inputs.gg_numpy(200_000, 1.0, 0.9, seed=5)
    f1 = oracle.fit(x)
    f2 = oracle.fit((x * np.float32(0.125)).astype(np.float32))  # exact power-of-two scaling
    assert f2.beta == pytest.approx(f1.beta, rel=1e-12)
    assert f2.alpha == pytest.approx(f1.alpha * 0.125, rel=1e-12)


# ---- Eq. 5: GG initialisation scale ------------------------------------------------------------
@pytest.mark.parametrize("d_in,xi", [(4096, 1.0), (11008, 2.0), (768, 2.0 / (1 + 0.01 ** 2))])
def test_init_alpha_reduces_to_he_at_shape_2(d_in, xi):
    # shape 2: Gamma(1/2)/Gamma(3/2) = 2 so alpha = sqrt(2 xi/d_in) and the variance alpha^2/2 = xi/d_in
    a = oracle.init_alpha(d_in, 2.0, xi)
    assert a == pytest.approx(math.sqrt(2.0 * xi / d_in), rel=1e-13)
    assert a * a / 2.0 == pytest.approx(xi / d_in, rel=1e-13)


@pytest.mark.parametrize("shape", [0.1, 0.5, 1.0, 2.0])
def test_init_alpha_gives_variance_xi_over_din(shape):
    # whatever the shape, the variance of GG(0, alpha, shape) (integrated from Eq. 1) must be xi/d_in
    d_in, xi = 1024, 2.0
    a = oracle.init_alpha(d_in, shape, xi)
    assert quad_moment(2, a, shape) == pytest.approx(xi / d_in, rel=1e-8)


def test_compression_ratio_matches_paper_tables():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_tables_compression.txt")
    rows = [tuple(map(float, l.split())) for l in open(path) if not l.startswith("#") and l.strip()]
    assert len(rows) == 24
    for eg, fl, c_pct in rows:
        assert 100.0 * oracle.compression_ratio(eg, fl) == pytest.approx(c_pct, abs=0.0051)
