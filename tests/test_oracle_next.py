"""Pins of the oracle's follow-on pieces: the GCT element-wise update (Algorithm 2), the
Exp-Golomb bit stream, and the Huffman mean length (the HM column of the result tables)."""
import heapq
import math

import numpy as np
import pytest

import gg_inputs
import oracle


# ---- GCT update ---------------------------------------------------------------------------------
def _state(n=5000, seed=0):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(n).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    gp = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    return w, g, gp


def test_gct_first_step_is_plain_sgd():
    w, g, gp = _state()
    w0 = w.copy()
    oracle.gct_update(w, g, gp, eta=1e-2, lam=0.5, eps=1e-8, inv_delta=2.0 ** 12, eg_k=0, n_rate=w.size,
                      first_step=True)
    assert np.array_equal(gp, g)                                   # equivalent gradient = gradient (h = 0)
    expect = (w0.astype(np.float64) - float(np.float32(1e-2)) * g.astype(np.float64)).astype(np.float32)
    assert np.array_equal(w, expect)


def test_gct_zero_lambda_is_plain_sgd():
    w, g, gp = _state(seed=1)
    w0 = w.copy()
    oracle.gct_update(w, g, gp, eta=1e-2, lam=0.0, eps=1e-8, inv_delta=2.0 ** 12, eg_k=0, n_rate=w.size,
                      first_step=False)
    assert np.array_equal(gp, g)
    expect = (w0.astype(np.float64) - float(np.float32(1e-2)) * g.astype(np.float64)).astype(np.float32)
    assert np.array_equal(w, expect)


def test_gct_step_by_hand():
    # one element, numbers chosen by hand: g = 3/1024, ghat_prev = 1/256, eps = 0, eta = 1/2, 2^n = 1024, k = 0
    w = np.array([1.0], dtype=np.float32)
    g = np.array([3.0 / 1024], dtype=np.float32)
    gp = np.array([1.0 / 256], dtype=np.float32)
    lam, N = 0.25, 10
    oracle.gct_update(w, g, gp, eta=0.5, lam=lam, eps=0.0, inv_delta=1024.0, eg_k=0, n_rate=N, first_step=False)
    h = (1 / 0.5) * (1 - (3 / 1024) / (1 / 256))                   # secant curvature of Eq. 5 / Algorithm 2
    q = 3                                                          # floor(3/1024 * 1024)
    u = 2 * q - 1                                                  # Map
    dR = 2.0 ** (10 + 2) / (N * math.log(2)) * 1.0 / (u + 1)       # rate gradient with the 2^k term restored
    ghat = 3 / 1024 + lam * dR * h
    assert gp[0] == pytest.approx(ghat, rel=1e-6)
    assert w[0] == pytest.approx(1.0 - 0.5 * ghat, rel=1e-6)


def test_gct_eps_guards_a_vanished_previous_gradient():
    # ghat_prev = 0: the secant curvature is (1/eta)(1 - g/eps), finite only through eps (Algorithm 2)
    w = np.array([0.5], dtype=np.float32)
    g = np.array([-5.0 / 256], dtype=np.float32)
    gp = np.zeros(1, dtype=np.float32)
    lam, N, eps = 0.125, 4, 2.0 ** -6
    oracle.gct_update(w, g, gp, eta=0.25, lam=lam, eps=eps, inv_delta=256.0, eg_k=1, n_rate=N, first_step=False)
    h = (1 / 0.25) * (1 - (-5 / 256) / eps)                        # = 4 * (1 + 1.25) = 9
    u = 2 * 5                                                      # floor(-5) = -5 -> Map = 10
    dR = 4 * 256 / (N * math.log(2)) * -1.0 / (u + 2)              # k = 1
    ghat = -5 / 256 + lam * dR * h
    assert h == 9.0
    assert gp[0] == pytest.approx(ghat, rel=1e-6)
    assert w[0] == pytest.approx(0.5 - 0.25 * ghat, rel=1e-6)


def test_gct_rate_gradient_is_slope_of_smoothed_eg_length():
    # d/dg of (1/N) * 2 log2(2 |g| 2^n + 2^k) at large |g| approaches the oracle's dR (u ~ 2|q|)
    n, k, N = 12, 0, 1000
    g0 = 0.37
    w = np.zeros(1, dtype=np.float32)
    g = np.array([g0], dtype=np.float32)
    gp = np.array([2 * g0], dtype=np.float32)       # with eps = 0: h = (1/eta)(1 - 1/2) = 1/(2 eta)
    eta, lam = 0.5, 1.0
    oracle.gct_update(w, g, gp, eta=eta, lam=lam, eps=0.0, inv_delta=2.0 ** n, eg_k=k, n_rate=N, first_step=False)
    dR = (float(gp[0]) - float(g[0])) / (lam * (1 / (2 * eta)))
    smooth = lambda v: 2.0 * math.log2(2.0 * abs(v) * 2 ** n + 2 ** k) / N
    fd = (smooth(g0 * 1.0001) - smooth(g0 * 0.9999)) / (g0 * 0.0002)
    assert dR == pytest.approx(fd, rel=2e-3)


# ---- Exp-Golomb bit stream ----------------------------------------------------------------------
@pytest.mark.parametrize("k", [0, 1, 3])
def test_eg_stream_round_trip_and_length(k):
    x = gg_inputs.gg_numpy(20_000, 0.02, 0.7, seed=3)
    r, _, sym = oracle.quantize_rate(x, 0.02 / 16, eg_k=k, want_symbols=True)
    u = np.array([oracle.map_symbol(int(q)) for q in sym], dtype=np.uint32)
    buf, nbits = oracle.eg_encode(u, k)
    assert nbits == r.eg_bits                                   # the rate estimate is the true stream size
    assert np.array_equal(oracle.eg_decode(buf, nbits, k, u.size), u)


def test_eg_stream_known_bits():
    buf, nbits = oracle.eg_encode(np.array([0, 1, 2, 3], dtype=np.uint32), 0)
    # codewords: 1 | 010 | 011 | 00100  -> 1010 0110 0100 (12 bits)
    assert nbits == 12 and list(buf) == [0b10100110, 0b01000000]


# ---- Huffman mean length ------------------------------------------------------------------------
def heap_huffman_mean(counts):
    h = [int(c) for c in counts if c]
    if len(h) == 1:
        return 1.0
    total = sum(h)
    heapq.heapify(h)
    coded = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        coded += a + b
        heapq.heappush(h, a + b)
    return coded / total


def test_dequantize_gives_the_lower_end_of_the_quantiser_cell():
    # hand values; the product is one fp32 rounding
    assert oracle.dequantize(np.array([-3, 0, 5, -(1 << 30)]), 0.25).tolist() == [-0.75, 0.0, 1.25, -float(1 << 28)]
    third = np.float32(1.0 / 3.0)
    assert oracle.dequantize(np.array([7]), float(third))[0] == np.float32(7) * third
    assert oracle.dequantize(np.array([16777217]), 2.0)[0] == 2.0 * 16777216.0          # q itself rounds to fp32 first
    # with the floor quantiser of Sec. 4.2 and an exact (power of two) step: q Delta <= x < (q + 1) Delta
    x = gg_inputs.gg_numpy(20_000, 0.02, 0.9, seed=4).astype(np.float32)
    delta = 2.0 ** -9
    _, _, q = oracle.quantize_rate(x, delta, want_symbols=True)
    lo = oracle.dequantize(q, delta)
    assert np.all(lo <= x) and np.all(x < lo + np.float32(delta))
    _, _, q_again = oracle.quantize_rate(lo, delta, want_symbols=True)
    assert np.array_equal(q_again, q)                                  # decoding and quantising again is the identity on symbols
    # nearest mode: within half a step
    _, _, qn = oracle.quantize_rate(x, delta, round_mode=oracle.ROUND_NEAREST_EVEN, want_symbols=True)
    assert np.all(np.abs(oracle.dequantize(qn, delta) - x) <= np.float32(delta / 2))
    # accumulate: one fp32 add onto what is there
    base = np.linspace(-1, 1, q.size, dtype=np.float32)
    acc = oracle.dequantize(q, delta, out=base.copy(), accumulate=True)
    assert np.array_equal(acc, base + lo)


def test_huffman_textbook_and_bounds():
    assert oracle.huffman_mean_bits(np.array([1, 1, 2, 4], dtype=np.uint64)) == pytest.approx((3 + 3 + 2 * 2 + 4) / 8)
    assert oracle.huffman_mean_bits(np.array([5, 5, 5, 5], dtype=np.uint64)) == 2.0
    assert oracle.huffman_mean_bits(np.array([0, 9, 0], dtype=np.uint64)) == 1.0
    for beta, seed in [(0.5, 1), (1.0, 2), (2.0, 3)]:
        x = gg_inputs.gg_numpy(200_000, 0.02, beta, seed=seed)
        r, hist, _ = oracle.quantize_rate(x, 0.02 / 16, nbins=65536)
        hm = oracle.huffman_mean_bits(hist)
        assert hm == pytest.approx(heap_huffman_mean(hist), rel=1e-12)
        assert r.entropy_bits <= hm < r.entropy_bits + 1          # Shannon bound for an optimal prefix code
        assert hm <= r.eg_bits / r.n + 1e-12                      # EG is one particular prefix code


# ---- rate gradient (ACT backward) ---------------------------------------------------------------
def test_rate_grad_is_slope_of_smoothed_mean_eg_length():
    n_exp, k, N = 10, 0, 500
    inv = 2.0 ** n_exp
    x = np.array([0.37, -0.9, 0.051, -0.0042, 3.3], dtype=np.float32)
    g = oracle.rate_grad(x, inv, k, N)
    smooth = lambda v: 2.0 * math.log2(2.0 * abs(v) * inv + 2 ** k) / N     # u ~ 2|x| 2^n
    for xi, gi in zip(x.astype(np.float64), g):
        fd = (smooth(xi * 1.0001) - smooth(xi * 0.9999)) / (xi * 0.0002)
        assert gi == pytest.approx(fd, rel=0.02 if abs(xi) * inv > 20 else 0.3)
    # printed form of Sec. 4.3 at k = 0 for a positive symbol: 2^(n+2)/(N ln 2) / (u + 1)
    q = math.floor(0.37 * inv)
    assert g[0] == pytest.approx(2.0 ** (n_exp + 2) / (N * math.log(2)) / (2 * q - 1 + 1), rel=1e-6)


def test_rate_grad_sign_zero_scale_accumulate_and_gct_consistency():
    x = np.array([0.0, -0.0, 0.25, -0.25, 1e-9, -1e-9], dtype=np.float32)
    g = oracle.rate_grad(x, 64.0, 1, 6)
    assert g[0] == 0 and g[1] == 0 and g[2] > 0 and g[3] < 0
    # floor puts -0.25*64 = -16 at u = 32 and +0.25*64 = 16 at u = 31: asymmetric by design
    assert g[2] == pytest.approx(4 * 64 / (6 * math.log(2)) / (31 + 2), rel=1e-6)
    assert g[3] == pytest.approx(-4 * 64 / (6 * math.log(2)) / (32 + 2), rel=1e-6)
    assert g[4] == pytest.approx(4 * 64 / (6 * math.log(2)) / 2, rel=1e-6)        # u = 0
    assert g[5] == pytest.approx(-4 * 64 / (6 * math.log(2)) / (2 + 2), rel=1e-6)  # q = -1 -> u = 2
    g2 = oracle.rate_grad(x, 64.0, 1, 6, scale=0.5)
    assert np.allclose(g2, 0.5 * g, rtol=1e-6)
    base = np.ones(6, dtype=np.float32)
    acc = oracle.rate_grad(x, 64.0, 1, 6, grad=base.copy(), accumulate=True)
    assert np.array_equal(acc, (base + g).astype(np.float32))
    # the GCT update uses the same rate gradient: with h = 1/(2 eta) (ghat_prev = 2g, eps = 0), ghat - g = lambda dR / (2 eta)
    gvec = np.array([0.37, -0.2], dtype=np.float32)
    w = np.zeros(2, dtype=np.float32)
    gp = (2 * gvec).astype(np.float32)
    oracle.gct_update(w, gvec, gp, eta=0.5, lam=1.0, eps=0.0, inv_delta=64.0, eg_k=1, n_rate=6, first_step=False)
    dr = oracle.rate_grad(gvec, 64.0, 1, 6)
    assert np.allclose(gp - gvec, dr, rtol=1e-5)
