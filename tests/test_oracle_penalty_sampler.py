"""Pins of the oracle's GG-prior penalty gradient, Philox4x32-10 and the Gamma-based GG sampler."""
import math
import os

import numpy as np
import pytest
from scipy import stats

import gg_inputs
import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---- penalty gradient: lambda d/dw (|w|/alpha)^beta, from the exponent of Eq. 1 -----------------
def test_penalty_laplace_and_gaussian_closed_forms():
    w = np.array([-3.0, -0.25, 0.5, 2.0, 1e-3], dtype=np.float32)
    alpha, lam = np.float32(0.5), np.float32(1e-2)
    g = oracle.penalty_grad(w, alpha, 1.0, lam)      # beta = 1: lambda sign(w)/alpha
    assert np.array_equal(g, (np.sign(w) * np.float32(float(lam) / float(alpha))).astype(np.float32))
    g = oracle.penalty_grad(w, alpha, 2.0, lam)      # beta = 2: 2 lambda w / alpha^2
    expect = (2.0 * float(lam) * w.astype(np.float64) / float(alpha) ** 2).astype(np.float32)
    assert np.array_equal(g, expect)


@pytest.mark.parametrize("beta", [0.5, 0.8, 1.3, 1.7, 3.0])
def test_penalty_is_derivative_of_prior_exponent(beta):
    alpha, lam = 0.02, 1e-4
    a32, b32, l32 = float(np.float32(alpha)), float(np.float32(beta)), float(np.float32(lam))
    w = np.array([-0.07, -0.02, -0.003, 0.001, 0.013, 0.05], dtype=np.float32)
    g = oracle.penalty_grad(w, alpha, beta, lam).astype(np.float64)
    cost = lambda v: l32 * (abs(v) / a32) ** b32
    for wi, gi in zip(w.astype(np.float64), g):
        h = abs(wi) * 1e-5
        fd = (cost(wi + h) - cost(wi - h)) / (2 * h)
        assert gi == pytest.approx(fd, rel=1e-6)


def test_penalty_zero_odd_symmetry_accumulate_bf16():
    w = np.array([0.0, -0.0, 0.3, -0.3], dtype=np.float32)
    for beta in (0.5, 1.0, 2.5):
        g = oracle.penalty_grad(w, 0.1, beta, 1e-3)
        assert g[0] == 0.0 and g[1] == 0.0          # sign(0) = 0 even where the limit diverges (beta < 1)
        assert g[2] == -g[3] and g[2] > 0
    base = np.array([1.0, -2.0, 0.5, 0.25], dtype=np.float32)
    acc = oracle.penalty_grad(w, 0.1, 1.5, 1e-3, grad=base.copy(), accumulate=True)
    assert np.array_equal(acc, base + oracle.penalty_grad(w, 0.1, 1.5, 1e-3))
    wb = gg_inputs.f32_to_bf16_bits(np.array([0.5, -0.125], dtype=np.float32))
    assert np.array_equal(oracle.penalty_grad(wb, 0.1, 1.5, 1e-3),
                          oracle.penalty_grad(np.array([0.5, -0.125], dtype=np.float32), 0.1, 1.5, 1e-3))


# ---- Philox4x32-10 ------------------------------------------------------------------------------
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if not l.startswith("#") and l.strip()]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_philox_words_look_uniform():
    words = np.array([oracle.philox4x32_10([0, 7, i, 0], [123, 456]) for i in range(20000)], dtype=np.uint64)
    for col in range(4):
        cnt = np.bincount((words[:, col] >> 28).astype(np.int64), minlength=16)
        chi2 = float(((cnt - 1250.0) ** 2 / 1250.0).sum())
        assert chi2 < 15 + 6 * math.sqrt(30)
    bits = ((words[:, 0, None] >> np.arange(32, dtype=np.uint64)) & 1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 0.02)
    a = words[:-1, 0].astype(np.float64)
    b = words[1:, 0].astype(np.float64)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.03


# ---- sampler ------------------------------------------------------------------------------------
N = 400_000


def test_sampler_laplace_case_is_exponential():
    x = oracle.sample(N, 0.02, 1.0, seed=5).astype(np.float64)
    assert stats.kstest(np.abs(x) / 0.02, "expon").pvalue > 1e-3


def test_sampler_gaussian_case_is_normal():
    alpha = 0.3
    x = oracle.sample(N, alpha, 2.0, seed=6).astype(np.float64)
    assert stats.kstest(x, "norm", args=(0.0, alpha / math.sqrt(2.0))).pvalue > 1e-3


@pytest.mark.parametrize("beta", [0.1, 0.5, 0.8, 1.5, 4.0])
def test_sampler_general_shape_transforms_to_gamma(beta):
    alpha = 0.015
    x = oracle.sample(N, alpha, beta, seed=7).astype(np.float64)
    g = (np.abs(x) / float(np.float32(alpha))) ** beta
    assert stats.kstest(g, "gamma", args=(1.0 / beta,)).pvalue > 1e-3
    assert abs((x > 0).mean() - 0.5) < 4 * 0.5 / math.sqrt(N)
    # independent check against scipy's generalized normal as a whole
    assert stats.kstest(x, "gennorm", args=(beta, 0.0, float(np.float32(alpha)))).pvalue > 1e-3


@pytest.mark.parametrize("beta", [0.1, 0.5, 1.0, 2.0, 4.0])
def test_sampler_rejection_step_has_the_published_efficiency(beta):
    """Marsaglia & Tsang (2000): with c = 1/sqrt(9 d) the normal envelope touches the transformed Gamma
    density exp(d ln v - d v + d), v = (1 + c z)^3, at z = 0 and lies above it elsewhere, so an attempt is
    accepted with probability P = (2 pi)^(-1/2) * integral of that density over 1 + c z > 0: above 0.95 for
    every shape >= 1.  A wrong c or d, or a wrong acceptance test, leaves the distribution tests above a chance
    (any envelope above the target still samples exactly) but not this count."""
    from scipy import integrate
    a = 1.0 / beta
    d = (a + 1.0 if a < 1.0 else a) - 1.0 / 3.0
    c = 1.0 / math.sqrt(9.0 * d)
    area, _ = integrate.quad(lambda z: math.exp(d * (3.0 * math.log1p(c * z) - (1.0 + c * z) ** 3 + 1.0)),
                             -1.0 / c, np.inf)
    p_accept = area / math.sqrt(2.0 * math.pi)
    assert 0.95 < p_accept < 1.0
    n = 200_000
    mean_attempts = oracle.sample_attempts(n, beta, seed=21) / n
    sigma = math.sqrt(1.0 - p_accept) / p_accept / math.sqrt(n)      # geometric number of attempts
    assert abs(mean_attempts - 1.0 / p_accept) < 5.0 * sigma
    # the draws are the ones sample() makes: the count does not depend on alpha, and is additive over ranges
    assert oracle.sample_attempts(1000, beta, seed=21) + oracle.sample_attempts(n - 1000, beta, seed=21, offset=1000) \
        == oracle.sample_attempts(n, beta, seed=21)


def test_sampler_fit_round_trip_and_variance_eq3():
    for alpha, beta in [(0.02, 1.0), (0.015, 1.5), (0.5, 0.8)]:
        x = oracle.sample(2_000_000, alpha, beta, seed=8)
        f = oracle.fit(x)
        assert abs(f.beta - beta) < 0.02 and f.alpha == pytest.approx(alpha, rel=0.01)
        var = alpha ** 2 * math.gamma(3 / beta) / math.gamma(1 / beta)
        assert float(np.mean(x.astype(np.float64) ** 2)) == pytest.approx(var, rel=0.01)


def test_sampler_is_a_pure_function_of_seed_stream_index():
    a = oracle.sample(1000, 0.1, 0.7, seed=99, stream=3, offset=0)
    b = oracle.sample(400, 0.1, 0.7, seed=99, stream=3, offset=600)
    assert np.array_equal(a[600:], b)
    c = oracle.sample(1000, 0.1, 0.7, seed=99, stream=4)
    d = oracle.sample(1000, 0.1, 0.7, seed=100, stream=3)
    assert not np.array_equal(a, c) and not np.array_equal(a, d)
    big = oracle.sample(4, 0.1, 0.7, seed=99, stream=3, offset=(1 << 32) - 2)
    lo = oracle.sample(2, 0.1, 0.7, seed=99, stream=3, offset=(1 << 32))
    assert np.array_equal(big[2:], lo)              # the index carries into the high counter word
    assert not np.array_equal(big[:2], lo)


def test_sampler_bf16_is_rounded_fp32():
    a = oracle.sample(5000, 0.1, 1.2, seed=1)
    b = oracle.sample(5000, 0.1, 1.2, seed=1, dtype=oracle.BF16)
    assert np.array_equal(b, gg_inputs.f32_to_bf16_bits(a))


def test_bf16_rounding_is_nearest_even():
    """Ties go to the even mantissa, in both directions; otherwise nearest; checked against the hand cases and
    against torch's own conversion on random values, ties, infinities and denormals."""
    import torch
    hand = {1.0 + 2.0 ** -8: 0x3F80,            # tie between 1.0 (even) and 1.0078125 -> down
            1.0 + 3 * 2.0 ** -8: 0x3F82,        # tie between 1.0078125 (odd) and 1.015625 -> up
            1.0 + 2.0 ** -8 + 2.0 ** -20: 0x3F81,   # just above the tie -> up
            -(1.0 + 2.0 ** -8): 0xBF80, 0.0: 0x0000, float("inf"): 0x7F80,
            3.3895314e38: 0x7F7F,               # the largest bf16 stays
            3.4028235e38: 0x7F80}               # the largest fp32 rounds up to infinity
    got = oracle.round_bf16(np.array(list(hand), dtype=np.float32))
    assert [int(v) for v in got] == list(hand.values())
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 1 << 32, size=200_000, dtype=np.uint64).astype(np.uint32)
    bits[:50_000] = (bits[:50_000] & np.uint32(0xFFFF0000)) | np.uint32(0x8000)      # exact ties
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.round_bf16(x), ref)
    nan = oracle.round_bf16(np.array([np.nan], dtype=np.float32))[0]
    assert (nan & 0x7F80) == 0x7F80 and (nan & 0x007F) != 0


def test_gg_init_sampling_has_he_variance():
    # Eq. 5 with shape 2 is He initialisation: variance xi/d_in
    d_in, xi = 4096, 2.0
    a = oracle.init_alpha(d_in, 2.0, xi)
    x = oracle.sample(1_000_000, a, 2.0, seed=12).astype(np.float64)
    assert x.var() == pytest.approx(xi / d_in, rel=0.01)
    a = oracle.init_alpha(d_in, 0.5, xi)
    x = oracle.sample(4_000_000, a, 0.5, seed=13).astype(np.float64)
    assert x.var() == pytest.approx(xi / d_in, rel=0.03)
