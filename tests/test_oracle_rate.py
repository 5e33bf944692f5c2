"""Pins of the oracle's quantiser, Map, Exp-Golomb length, histogram, entropy and bit count
(Sec. 4.2) against the paper's Map table, explicit codeword construction, exact rational
arithmetic, brute-force counting and the closed form for a Laplace source."""
import math
import os
from collections import Counter
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

import gg_inputs
import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---- Map ---------------------------------------------------------------------------------------
def test_map_paper_table():
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLD, "map_table.txt"))
            if not l.startswith("#") and l.strip()]
    assert len(rows) == 9
    for q, u in rows:
        assert oracle.map_symbol(q) == u


def test_map_bijection_parity_and_order():
    R = 1 << 16
    us = [oracle.map_symbol(q) for q in range(-R, R + 1)]
    assert sorted(us) == list(range(0, 2 * R + 1))          # bijection onto 0..2R
    for q, u in zip(range(-R, R + 1), us):
        if q > 0:
            assert u % 2 == 1 and (u + 1) // 2 == q          # positives odd
        elif q < 0:
            assert u % 2 == 0 and u // 2 == -q               # negatives even
        else:
            assert u == 0
    assert oracle.map_symbol(1 << 30) == (1 << 31) - 1
    assert oracle.map_symbol(-(1 << 30)) == 1 << 31


# ---- Exp-Golomb length: build the codeword and count its bits -----------------------------------
def eg_codeword(u: int, k: int) -> str:
    """Order-k Exp-Golomb: unary-coded quotient part then k suffix bits, built as a bit string."""
    v = u + (1 << k)
    binary = bin(v)[2:]
    return "0" * (len(binary) - 1 - k) + binary


def test_eg_len_hand_values():
    assert oracle.eg_len(0, 0) == 1
    assert oracle.eg_len(1, 0) == 3 and oracle.eg_len(2, 0) == 3
    assert [oracle.eg_len(u, 0) for u in range(3, 7)] == [5, 5, 5, 5]
    assert oracle.eg_len(7, 0) == 7
    assert eg_codeword(0, 0) == "1" and eg_codeword(1, 0) == "010" and eg_codeword(4, 0) == "00101"
    assert oracle.eg_len(0, 3) == 4                         # k suffix bits + the marker bit


@pytest.mark.parametrize("k", [0, 1, 2, 3, 4, 9, 15])
def test_eg_len_equals_codeword_length(k):
    us = list(range(0, 1 << 12)) + [(1 << 16) - 1, 1 << 16, (1 << 31) - 1, 1 << 31, (1 << 32) - 1]
    for u in us:
        assert oracle.eg_len(u, k) == len(eg_codeword(u, k)), (u, k)


def test_eg_code_is_prefix_free_kraft():
    for k in (0, 2):
        total = sum(Fraction(1, 2 ** oracle.eg_len(u, k)) for u in range(0, (1 << 10) - (1 << k)))
        # codewords of all u with u + 2^k < 2^10 fill the code tree down to that depth exactly
        assert total == 1 - Fraction(1, 2 ** (10 - k))


# ---- quantiser: floor semantics, exactness, edge cases -----------------------------------------
def test_quantize_power_of_two_step_is_exact_floor():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(4000) * 3).astype(np.float32)
    for n in (0, 3, 8):
        inv = float(2 ** n)
        for v in x:
            expect = math.floor(Fraction(float(v)) * 2 ** n)
            assert oracle.quantize_one(float(v), inv, oracle.ROUND_FLOOR) == expect


def test_quantize_dead_zone_is_asymmetric_under_floor():
    inv = 16.0  # Delta = 1/16
    assert oracle.quantize_one(0.0, inv) == 0
    assert oracle.quantize_one(-0.0, inv) == 0
    assert oracle.quantize_one(0.06, inv) == 0              # [0, Delta) -> 0
    assert oracle.quantize_one(-1e-30, inv) == -1           # [-Delta, 0) -> -1
    assert oracle.quantize_one(0.0625, inv) == 1
    assert oracle.quantize_one(-0.0625, inv) == -1
    assert oracle.quantize_one(-0.0626, inv) == -2


def test_quantize_keeps_denormals():
    tiny = float(np.float32(1e-45))  # smallest positive denormal
    assert oracle.quantize_one(-tiny, 1.0) == -1
    assert oracle.quantize_one(tiny, 1.0) == 0
    # product that is denormal: (-2^-100) * 2^-40 = -2^-140
    assert oracle.quantize_one(-(2.0 ** -100), 2.0 ** -40) == -1


def test_quantize_nan_inf_and_clamp():
    assert oracle.quantize_one(float("nan"), 4.0) == 0
    assert oracle.quantize_one(float("inf"), 4.0) == 1 << 30
    assert oracle.quantize_one(float("-inf"), 4.0) == -(1 << 30)
    assert oracle.quantize_one(3e9, 1.0) == 1 << 30
    assert oracle.quantize_one(-3e9, 1.0) == -(1 << 30)
    assert oracle.quantize_one(0.0, float("inf")) == 0      # 0 * inf = NaN -> 0
    r, _, _ = oracle.quantize_rate(np.array([np.nan, 1.0], dtype=np.float32), 1.0)
    assert r.flags & oracle.NONFINITE
    r, _, _ = oracle.quantize_rate(np.array([1e30, 1.0], dtype=np.float32), 1.0)
    assert r.flags & oracle.SATURATED and r.u_max == (1 << 31) - 1 and r.fl_bits == 31


def test_quantize_nearest_even_mode():
    for v, e in [(0.5, 0), (1.5, 2), (2.5, 2), (-0.5, 0), (-1.5, -2), (0.49, 0), (0.51, 1), (-2.5, -2)]:
        assert oracle.quantize_one(v, 1.0, oracle.ROUND_NEAREST_EVEN) == e


def test_quantize_uses_single_fp32_product():
    # x * inv rounded to fp32 differs from the double product for these operands
    x, delta = np.float32(0.1), np.float32(0.3)
    inv = np.float32(1.0) / delta
    t32 = np.float32(x * inv)
    assert oracle.quantize_one(float(x), float(inv)) == math.floor(float(t32))
    # a case where floor(fp32 product) != floor(exact quotient): x = 3*Delta exactly in fp32 terms
    d = np.float32(0.1)
    xs = (np.arange(1, 2000, dtype=np.float32) * d).astype(np.float32)
    r, _, sym = oracle.quantize_rate(xs, float(d), want_symbols=True)
    invd = np.float32(1.0) / d
    expect = np.floor((xs * invd).astype(np.float32)).astype(np.int64)
    assert np.array_equal(sym, expect)


# ---- histogram / bits / entropy: brute force ---------------------------------------------------
def brute(x, delta, k, nbins, mode="floor"):
    inv = np.float32(1.0) / np.float32(delta)
    t = (x.astype(np.float32) * inv).astype(np.float32)
    q = np.floor(t) if mode == "floor" else np.rint(t)
    q = q.astype(np.int64)
    u = np.where(q > 0, 2 * q - 1, -2 * q)
    bits = sum(len(eg_codeword(int(v), k)) for v in u)
    cnt = Counter(int(min(v, nbins - 1)) for v in u)
    n = len(u)
    H = -sum(c / n * math.log2(c / n) for c in cnt.values())
    return q, u, bits, cnt, H


@pytest.mark.parametrize("beta,delta_div,k,nbins", [(1.0, 16, 0, 4096), (0.6, 8, 0, 64), (2.0, 4, 2, 32),
                                                    (1.5, 32, 1, 1024)])
def test_rate_matches_brute_force(beta, delta_div, k, nbins):
    alpha = 0.02
    x = gg_inputs.gg_numpy(10_000, alpha, beta, seed=21)
    delta = np.float32(alpha) / np.float32(delta_div)
    r, hist, sym = oracle.quantize_rate(x, float(delta), eg_k=k, nbins=nbins, want_symbols=True)
    q, u, bits, cnt, H = brute(x, delta, k, nbins)
    assert np.array_equal(sym, q)
    assert r.eg_bits == bits and r.n == x.size and r.u_max == int(u.max())
    assert r.fl_bits == max(1, int(u.max()).bit_length())
    assert r.n_clamped == int((u > nbins - 1).sum())
    assert {b: int(c) for b, c in enumerate(hist) if c} == dict(cnt)
    assert int(hist.sum()) == x.size
    assert r.entropy_bits == pytest.approx(H, rel=1e-12)
    if r.n_clamped == 0:
        assert sum(int(c) * oracle.eg_len(b, k) for b, c in enumerate(hist)) == r.eg_bits
        assert r.entropy_bits <= r.eg_bits / r.n + 1e-12     # no prefix code beats the entropy
    assert r.entropy_bits <= math.log2(np.count_nonzero(hist)) + 1e-12


def test_rate_bf16_and_nearest_mode_match_brute_force():
    x = gg_inputs.gg_numpy(5000, 0.5, 0.8, seed=22)
    xb = gg_inputs.f32_to_bf16_bits(x)
    xw = gg_inputs.bf16_bits_to_f32(xb)
    delta = np.float32(0.5 / 8)
    r, hist, sym = oracle.quantize_rate(xb, float(delta), eg_k=0, round_mode=oracle.ROUND_NEAREST_EVEN,
                                        nbins=512, want_symbols=True)
    q, u, bits, cnt, H = brute(xw, delta, 0, 512, mode="nearest")
    assert np.array_equal(sym, q) and r.eg_bits == bits
    assert {b: int(c) for b, c in enumerate(hist) if c} == dict(cnt)


def test_rate_hand_cases():
    z = np.zeros(1000, dtype=np.float32)
    r, hist, _ = oracle.quantize_rate(z, 0.01, nbins=16)
    assert r.eg_bits == 1000 and r.entropy_bits == 0.0 and r.u_max == 0 and r.fl_bits == 1
    assert hist[0] == 1000 and hist[1:].sum() == 0
    # two equiprobable values: q in {0, 1} -> H = 1 bit, EG bits = 1 and 3
    x = np.tile(np.array([0.5, 1.5], dtype=np.float32), 500)
    r, hist, _ = oracle.quantize_rate(x, 1.0, nbins=16)
    assert r.entropy_bits == 1.0 and r.eg_bits == 500 * 1 + 500 * 3 and r.u_max == 1
    # empty
    r, _, _ = oracle.quantize_rate(np.zeros(0, dtype=np.float32), 1.0, nbins=4)
    assert r.n == 0 and r.eg_bits == 0 and r.flags & oracle.EMPTY and r.fl_bits == 1
    # overflow bin: symbols 0,1,2,3,4 with nbins 3 -> bin 2 holds u=2,3,4; two of them are clamped
    x = np.array([0.5, 1.5, -0.5, 2.5, -1.5], dtype=np.float32)  # q = 0,1,-1,2,-2 -> u = 0,1,2,3,4
    r, hist, _ = oracle.quantize_rate(x, 1.0, nbins=3)
    assert list(hist) == [1, 1, 3] and r.n_clamped == 2 and r.u_max == 4 and r.fl_bits == 3
    assert r.eg_bits == 1 + 3 + 3 + 5 + 5


# ---- Laplace source under the floor quantiser: closed form ---------------------------------------
def laplace_floor_probs(r, jmax=4000):
    """P(q = j) for x ~ Laplace(scale alpha), q = floor(x/Delta), r = Delta/alpha.
    j >= 0: (e^{-jr} - e^{-(j+1)r})/2 ; q = -j-1 has the same mass (mirror interval)."""
    j = np.arange(jmax, dtype=np.float64)
    p = 0.5 * (np.exp(-j * r) - np.exp(-(j + 1) * r))
    return j.astype(np.int64), p


def test_laplace_closed_form_entropy_and_eg_rate():
    r = 1.0 / 16.0
    j, p = laplace_floor_probs(r)
    # q = j -> u = 2j-1 (j>0), 0 (j=0);  q = -j-1 -> u = 2j+2
    u_pos = np.where(j > 0, 2 * j - 1, 0)
    u_neg = 2 * j + 2
    H = -2.0 * np.sum(p * np.log2(p))
    mean_len = float(np.sum(p * [oracle.eg_len(int(v), 0) for v in u_pos]) +
                     np.sum(p * [oracle.eg_len(int(v), 0) for v in u_neg]))
    # small-step law: H ~ h(X)/ln2 - log2(Delta), h = 1 + ln(2 alpha) for Laplace
    assert H == pytest.approx((1.0 + math.log(2.0)) / math.log(2.0) - math.log2(r), abs=5e-4)
    assert H == pytest.approx(6.44293, abs=2e-5)
    # the same mean with the order-0 length written out as 2 * bit_length(u + 1) - 1
    by_hand = float(np.sum(p * [2 * int(v + 1).bit_length() - 1 for v in u_pos]) + np.sum(p * [2 * int(v + 1).bit_length() - 1 for v in u_neg]))
    assert mean_len == pytest.approx(by_hand, abs=1e-12) and mean_len == pytest.approx(8.69872, abs=2e-5)
    # sampled source (scipy's Laplace, independent of the oracle's sampler)
    alpha, n = 0.02, 4_000_000
    x = stats.laplace.rvs(scale=alpha, size=n, random_state=np.random.default_rng(3)).astype(np.float32)
    rt, hist, _ = oracle.quantize_rate(x, float(np.float32(alpha) / np.float32(16)), nbins=4096)
    assert rt.n_clamped == 0
    assert rt.entropy_bits == pytest.approx(H, abs=3e-3)
    assert rt.eg_bits / n == pytest.approx(mean_len, abs=5e-3)
    # chi-square of the histogram against the closed-form cell probabilities (cells with >= 50 expected)
    expect = np.zeros(4096)
    np.add.at(expect, u_pos[u_pos < 4096], p[u_pos < 4096] * n)
    np.add.at(expect, u_neg[u_neg < 4096], p[u_neg < 4096] * n)
    m = expect >= 50
    chi2 = float(np.sum((hist[m].astype(np.float64) - expect[m]) ** 2 / expect[m]))
    dof = int(m.sum()) - 1
    assert chi2 < dof + 6.0 * math.sqrt(2.0 * dof)


# ---- segmented pass = per-segment calls ---------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True])
def test_fused_segmented_equals_per_segment_calls(bf16):
    sizes = [0, 17, 4096, 1, 3000, 0, 999]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    parts = [gg_inputs.gg_numpy(s, 10.0 ** (-2 - i % 3), 0.6 + 0.2 * i, seed=30 + i) for i, s in enumerate(sizes)]
    x = np.concatenate(parts).astype(np.float32)
    if bf16:
        x = gg_inputs.f32_to_bf16_bits(x)              # uint16 bit patterns: element offsets are 2-byte strides
    grad = np.zeros(x.size, dtype=np.float32)
    fits, rates = oracle.fused_segmented(x, off, delta_div=16.0, lam=1e-4, grad=grad)
    for s, sz in enumerate(sizes):
        xs = x[off[s]:off[s + 1]]
        f = oracle.fit(xs)
        assert (fits[s].n, fits[s].sum_abs, fits[s].sum_sq, fits[s].beta, fits[s].alpha, fits[s].flags) == \
               (f.n, f.sum_abs, f.sum_sq, f.beta, f.alpha, f.flags)
        if sz == 0:
            assert rates[s].flags & oracle.EMPTY and rates[s].eg_bits == 0
            continue
        if f.alpha == 0:
            continue
        delta = np.float32(f.alpha) / np.float32(16.0)
        r, _, _ = oracle.quantize_rate(xs, float(delta))
        assert (rates[s].eg_bits, rates[s].u_max, rates[s].fl_bits) == (r.eg_bits, r.u_max, r.fl_bits)
        g = oracle.penalty_grad(xs, np.float32(f.alpha), np.float32(f.beta), 1e-4)
        assert np.array_equal(grad[off[s]:off[s + 1]], g)
