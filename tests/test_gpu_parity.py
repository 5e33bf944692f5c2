"""GPU parity: libgg (through its C ABI, via the ctypes binding) against the CPU oracle, element
by element on the same seeded inputs.  Sizes span several 16384-element chunks and ragged tails."""
import math

import numpy as np
import pytest
import torch

import gg_inputs
import oracle
import parity
from parity import (check_fit, check_penalty, check_rate, host_bits)

pytestmark = pytest.mark.gpu

DEV = "cuda"


@pytest.fixture(scope="module")
def gg():
    import paper_2506_00486_amd as m
    m.lib()
    return m


def make(n, alpha, beta, seed, dtype=torch.float32):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    return gg_inputs.gg_torch(n, alpha, beta, gen, DEV, dtype)


SIZES = [0, 1, 3, 4, 5, 17, 255, 4095, 16384, 16385, 16384 * 3 + 7, 100_003, 1_048_576]


# ---- fit ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n", SIZES)
def test_fit_single_tensor(gg, n, dtype):
    print(f"fit n={n} dtype={dtype}", flush=True)
    x = make(n, 0.02, 1.0, seed=n + 1, dtype=dtype)
    ws = gg.Workspace(n, 1)
    rec = gg.fit_records(gg.gg_fit(x, ws))[0]
    check_fit(rec, oracle.fit(host_bits(x)), f"n={n}")


@pytest.mark.parametrize("alpha,beta,dtype,seed", [(0.02, 1.0, torch.float32, 0), (0.015, 1.5, torch.bfloat16, 1),
                                                   (0.5, 0.8, torch.bfloat16, 2), (3e-5, 0.5, torch.float32, 3),
                                                   (0.01, 2.0, torch.float32, 4), (1.0, 0.12, torch.float32, 5),
                                                   (1.0, 8.0, torch.float32, 6)])
def test_fit_recovers_shapes(gg, alpha, beta, dtype, seed):
    n = 1 << 21
    x = make(n, alpha, beta, seed, dtype)
    ws = gg.Workspace(n, 1)
    rec = gg.fit_records(gg.gg_fit(x, ws))[0]
    check_fit(rec, oracle.fit(host_bits(x)))
    assert abs(float(rec["beta"]) - beta) < (0.02 if beta <= 2 else 0.05 * beta)


def test_fit_unaligned_views_and_special_values(gg):
    base = make(70_000, 0.1, 1.2, seed=9)
    ws = gg.Workspace(70_000, 1)
    # the binding requires 16-byte aligned bases; element-index misalignment is exercised through segments
    off = [0, 1, 3, 6, 10, 16389, 16390, 40_001, 70_000]
    rec = gg.fit_records(gg.gg_fit_segmented(base, off, gg.Workspace(70_000, len(off) - 1)))
    hb = host_bits(base)
    for s in range(len(off) - 1):
        check_fit(rec[s], oracle.fit(hb[off[s]:off[s + 1]]), f"seg {s}")
    # degenerate / clamped / non-finite inputs
    for vals in ([0.0] * 100, [0.5, -0.5] * 50, [1.0, float("nan"), 2.0], [1.0, float("inf")],
                 [1e-15, -2e-16, 3e-17], [1.0] + [0.0] * 9999):
        x = torch.tensor(vals, dtype=torch.float32, device=DEV)
        rec1 = gg.fit_records(gg.gg_fit(x, ws))[0]
        check_fit(rec1, oracle.fit(host_bits(x)), str(vals[:3]))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fit_segmented_ragged_bucket(gg, dtype):
    segs = gg_inputs.scaled_layout(gg_inputs.gradient_bucket_1p5b()[:27] + gg_inputs.gradient_bucket_1p5b()[-1:], 997)
    segs.insert(5, gg_inputs.Segment("empty", 0))
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=3, device=DEV, dtype=dtype)
    ws = gg.Workspace(flat.numel(), len(segs))
    rec = gg.fit_records(gg.gg_fit_segmented(flat, off, ws))
    hb = host_bits(flat)
    for s in range(len(segs)):
        check_fit(rec[s], oracle.fit(hb[off[s]:off[s + 1]]), segs[s].name)


def test_bucket_of_thousands_of_small_units(gg):
    # 6000 units of 0 .. 40,000 elements (many shorter than a chunk, some empty, a few spanning several runs):
    # the many-unit finalisations (one lane per unit) and the unit search of the sweeps
    rng = np.random.default_rng(12)
    sizes = rng.integers(0, 600, size=6000)
    sizes[rng.integers(0, 6000, size=300)] = 0
    sizes[rng.integers(0, 6000, size=40)] = rng.integers(17_000, 40_000, size=40)
    sizes[:3] = (0, 1, 2)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = make(n, 0.01, 0.9, seed=77)
    ws = gg.Workspace(n, len(sizes))
    res = gg.gg_fused_segmented(x, off, ws, delta_div=16.0, want_symbols=True)
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    sym = res["symbols"].cpu().numpy()
    hb = host_bits(x)
    picks = list(range(0, 12)) + list(rng.integers(0, 6000, size=150)) + list(np.flatnonzero(sizes > 16_384)[:10]) + [5999]
    for s in picks:
        lo, hi = int(off[s]), int(off[s + 1])
        o = oracle.fit(hb[lo:hi])
        check_fit(frec[s], o, f"unit {s} ({hi - lo} elements)")
        d = float(rrec[s]["delta"])
        if hi == lo or not (d > 0 and np.isfinite(d)):
            assert int(rrec[s]["eg_bits"]) == 0
            continue
        r, _, osym = oracle.quantize_rate(hb[lo:hi], d, want_symbols=True)
        check_rate(rrec[s], r, f"unit {s}", entropy=False)
        assert np.array_equal(sym[lo:hi], osym)
    assert int(rrec["n"].astype(np.int64).sum()) == n


@pytest.mark.parametrize("rows,cols", [(7, 4096), (64, 1000), (3, 40_000), (1, 5), (5, 16384)])
def test_fit_rows_and_total(gg, rows, cols):
    x = make(rows * cols, 0.5, 0.8, seed=rows, dtype=torch.bfloat16)
    ws = gg.Workspace(rows * cols, rows)
    out, total = gg.gg_fit_rows(x, rows, cols, ws, want_total=True)
    rec, tot = gg.fit_records(out), gg.fit_records(total)[0]
    hb = host_bits(x)
    for r in range(rows):
        check_fit(rec[r], oracle.fit(hb[r * cols:(r + 1) * cols]), f"row {r}")
    check_fit(tot, oracle.fit(hb), "total")


def test_fit_is_reproducible(gg):
    x = make(3_000_001, 0.02, 0.9, seed=77)
    ws = gg.Workspace(x.numel(), 1)
    a = gg.gg_fit(x, ws).cpu().numpy().tobytes()
    b = gg.gg_fit(x, ws).cpu().numpy().tobytes()
    assert a == b


# ---- quantise + rate ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n", [0, 1, 5, 4099, 16384 * 2 + 3, 300_001])
@pytest.mark.parametrize("mode", [0, 1])
def test_quantize_rate_single(gg, n, dtype, mode):
    print(f"rate n={n} dtype={dtype} mode={mode}", flush=True)
    alpha = 0.02
    x = make(n, alpha, 1.0, seed=n + 5, dtype=dtype)
    delta = float(np.float32(alpha) / np.float32(16))
    ws = gg.Workspace(n, 1)
    for k, nbins in ((0, 0), (0, 4096), (2, 64)):
        out, hist, sym = gg.gg_quantize_rate(x, delta, ws, eg_k=k, round_mode=mode, nbins=nbins, want_symbols=True)
        rec = gg.rate_records(out)[0]
        r, ohist, osym = oracle.quantize_rate(host_bits(x), delta, eg_k=k, round_mode=mode, nbins=nbins,
                                              want_symbols=True)
        check_rate(rec, r, f"n={n} k={k} nbins={nbins}")
        assert float(rec["delta"]) == delta
        assert np.array_equal(sym.cpu().numpy(), osym)
        if nbins:
            assert np.array_equal(hist.cpu().numpy().view(np.uint64), ohist)


def test_quantize_special_values(gg):
    vals = [0.0, -0.0, 1e-45, -1e-45, -1e-40, 1e-40, float("nan"), float("inf"), float("-inf"), 3e9, -3e9, 0.5, -0.5,
            1.5, 2.5, -1.5, -2.5, 0.0625, -0.0625, 0.06, -0.0626, 1.0, -1.0, 123456.789, -(2.0 ** -100)]
    x = torch.tensor(vals * 3, dtype=torch.float32, device=DEV)
    ws = gg.Workspace(x.numel(), 1)
    for delta in (1.0, 0.0625, 2.0 ** 40, 1e-30):
        for mode in (0, 1):
            out, hist, sym = gg.gg_quantize_rate(x, delta, ws, eg_k=1, round_mode=mode, nbins=16, want_symbols=True)
            r, ohist, osym = oracle.quantize_rate(host_bits(x), delta, eg_k=1, round_mode=mode, nbins=16,
                                                  want_symbols=True)
            assert np.array_equal(sym.cpu().numpy(), osym), (delta, mode)
            check_rate(gg.rate_records(out)[0], r, f"delta={delta} mode={mode}")
            assert np.array_equal(hist.cpu().numpy().view(np.uint64), ohist)
            # the lean kernels (k = 0, no histogram, no symbols) take the code length from the float exponent
            out0, _, _ = gg.gg_quantize_rate(x, delta, ws, eg_k=0, round_mode=mode)
            r0, _, _ = oracle.quantize_rate(host_bits(x), delta, eg_k=0, round_mode=mode)
            check_rate(gg.rate_records(out0)[0], r0, f"lean delta={delta} mode={mode}", entropy=False)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("mode", [0, 1])
def test_lean_rate_kernel_matches_integer_path(gg, dtype, mode):
    """k = 0 without histogram/symbols uses exponent-derived lengths; every power-of-two boundary of |q| and
    both signs must give the same bit count and u_max as the integer path and the oracle."""
    edges = []
    for e in range(0, 31):
        for d in (-1.0, -0.5, 0.0, 0.5, 1.0):
            edges += [2.0 ** e + d, -(2.0 ** e) + d]
    base = torch.tensor(edges, dtype=torch.float32, device=DEV).to(dtype)
    rnd = make(200_000, 40.0, 0.6, seed=31, dtype=dtype)             # symbols spread over ~2^20
    x = torch.cat([base, rnd, torch.zeros(777, device=DEV, dtype=dtype), base * 0.001]).contiguous()
    ws = gg.Workspace(x.numel(), 1)
    for delta in (1.0, 0.37, 2.0 ** -9):
        lean, _, _ = gg.gg_quantize_rate(x, delta, ws, eg_k=0, round_mode=mode)
        full, _, _ = gg.gg_quantize_rate(x, delta, ws, eg_k=0, round_mode=mode, want_symbols=True)
        a, b = gg.rate_records(lean)[0], gg.rate_records(full)[0]
        r, _, _ = oracle.quantize_rate(host_bits(x), delta, eg_k=0, round_mode=mode)
        check_rate(a, r, f"lean delta={delta}", entropy=False)
        check_rate(b, r, f"full delta={delta}", entropy=False)
        # the sweep that also writes the penalty gradient takes the exponent path too (short blocks, a slot each)
        n = x.numel()
        grad = torch.empty(n, dtype=torch.float32, device=DEV)
        out = gg.gg_fused_segmented(x, [0, n], ws, delta_div=0.0, delta=torch.tensor([delta], dtype=torch.float32, device=DEV),
                                    eg_k=0, round_mode=mode, lam=1e-3, grad=grad)
        check_rate(gg.rate_records(out["rate"])[0], r, f"with penalty delta={delta}", entropy=False)
        f = gg.fit_records(out["fit"])[0]
        want = oracle.penalty_grad(host_bits(x), float(f["alpha"]), float(f["beta"]), 1e-3)
        check_penalty(grad.cpu().numpy(), want, f"penalty beside the lean rate, delta={delta}")


def test_solver_alone_from_the_kernel_s_own_moments(gg):
    # the moment sums read back from the GPU record go through the oracle's solver: what is left is the
    # difference of the two root finders (64-way bracketing + inverse cubic vs 200-step bisection)
    # and the rounding of beta, alpha to fp32
    shapes = [0.06, 0.1, 0.3, 0.5, 0.8, 1.0, 1.5, 2.0, 3.0, 7.0, 15.0, 19.0]
    sizes = [200_000] * len(shapes)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    x = torch.cat([make(n, 0.01 * (i + 1), b, seed=100 + i) for i, (n, b) in enumerate(zip(sizes, shapes))])
    for S_units, fit in ((len(shapes), gg.gg_fit_segmented(x, off, gg.Workspace(x.numel(), len(shapes)))),):
        rec = gg.fit_records(fit)
        for s in range(S_units):
            o = oracle.fit_from_moments(float(rec[s]["sum_abs"]), float(rec[s]["sum_sq"]), int(rec[s]["n"]))
            assert int(rec[s]["flags"]) == o.flags
            assert abs(float(rec[s]["beta"]) - o.beta) <= 2e-7 * o.beta, (s, rec[s], o)
            assert abs(float(rec[s]["alpha"]) - o.alpha) <= 2e-7 * o.alpha, (s, rec[s], o)
    # single tensor (wave solver) and a many-unit call (tabulated curve): same bar
    one = gg.fit_records(gg.gg_fit(x[:200_000], gg.Workspace(200_000, 1)))[0]
    o = oracle.fit_from_moments(float(one["sum_abs"]), float(one["sum_sq"]), int(one["n"]))
    assert abs(float(one["beta"]) - o.beta) <= 2e-7 * o.beta and abs(float(one["alpha"]) - o.alpha) <= 2e-7 * o.alpha
    rows, cols = 4800, 500
    fr = gg.fit_records(gg.gg_fit_rows(x, rows, cols, gg.Workspace(x.numel(), rows)))
    for r in range(0, rows, 97):
        o = oracle.fit_from_moments(float(fr[r]["sum_abs"]), float(fr[r]["sum_sq"]), int(fr[r]["n"]))
        assert abs(float(fr[r]["beta"]) - o.beta) <= 2e-7 * o.beta, (r, fr[r], o)
        assert abs(float(fr[r]["alpha"]) - o.alpha) <= 2e-7 * o.alpha, (r, fr[r], o)


def test_histogram_beyond_lds_bins_and_overflow_bin(gg):
    # activation-like: heavy tail with outliers; symbols far above the LDS-resident bins and above nbins
    x = gg_inputs.make_tensor((300_000,), 0.5, 0.8, seed=2, device=DEV, dtype=torch.bfloat16, outlier_frac=1e-3,
                              outlier_scale=20.0)
    ws = gg.Workspace(x.numel(), 1)
    # 12288 block-private bins: the clamping bin sits just inside, on and beyond that boundary
    for nbins, div in ((32768, 64), (65536, 512), (20000, 512), (12289, 512), (12288, 512), (1000, 8), (2, 8)):
        delta = float(np.float32(0.5) / np.float32(div))
        out, hist, _ = gg.gg_quantize_rate(x, delta, ws, nbins=nbins)
        r, ohist, _ = oracle.quantize_rate(host_bits(x), delta, nbins=nbins)
        check_rate(gg.rate_records(out)[0], r, f"nbins={nbins}")
        assert np.array_equal(hist.cpu().numpy().view(np.uint64), ohist)
    assert r.n_clamped > 0


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_histogram_beside_symbols_and_penalty_in_short_and_resident_blocks(gg, dtype, mode):
    """A histogram together with a written stream: buckets of a few chunks run as short blocks with 4096 private
    bins, larger ones as resident runs with 12288.  Both against the oracle, with symbols beyond the private bins
    and beyond the histogram, NaN / Inf / zeros, empty units, both rounding modes."""
    for sizes in ([5000, 0, 70_000, 16384, 1, 250_000, 4097], [3_400_000, 0, 50_000, 1000]):
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        n, S = int(off[-1]), len(sizes)
        x = gg_inputs.make_tensor((n,), 0.5, 0.8, seed=21 + S, device=DEV, dtype=dtype, outlier_frac=1e-3, outlier_scale=20.0)
        x[off[-2] + 3] = float("nan"); x[off[2] + 5] = float("inf"); x[off[2] + 6] = -float("inf"); x[off[3]: off[3] + 300] = 0
        hb = host_bits(x)
        ws = gg.Workspace(n, S)
        for nbins, div in ((300, 64.0), (4096, 256.0), (4097, 256.0), (20000, 1024.0)):
            grad = torch.full((n,), 7.0, dtype=torch.float32, device=DEV)
            clamped, largest = 0, 0
            out = gg.gg_fused_segmented(x, off, ws, delta_div=div, eg_k=1, round_mode=mode, nbins=nbins, want_symbols=True,
                                        lam=1e-3, grad=grad)
            frec, rrec = gg.fit_records(out["fit"]), gg.rate_records(out["rate"])
            hist = out["hist"].cpu().numpy().view(np.uint64).reshape(S, nbins)
            sym, g = out["symbols"].cpu().numpy(), grad.cpu().numpy()
            for s in range(S):
                lo, hi = int(off[s]), int(off[s + 1])
                if hi == lo:
                    assert rrec[s]["flags"] == gg.GG_F_EMPTY and not hist[s].any()
                    continue
                if rrec[s]["flags"] & gg.GG_F_DEGENERATE:       # a unit whose fit saw NaN / Inf has no step (the last one and unit 2)
                    assert s in (2, S - 1)
                    assert not hist[s].any() and not sym[lo:hi].any()
                    continue
                r, ohist, osym = oracle.quantize_rate(hb[lo:hi], float(rrec[s]["delta"]), eg_k=1, round_mode=mode, nbins=nbins,
                                                      want_symbols=True)
                check_rate(rrec[s], r, f"sizes={sizes[:2]} nbins={nbins} seg {s}")
                clamped += r.n_clamped; largest = max(largest, r.u_max)
                assert np.array_equal(hist[s], ohist) and np.array_equal(sym[lo:hi], osym), (nbins, s)
                og = oracle.penalty_grad(hb[lo:hi], float(frec[s]["alpha"]), float(frec[s]["beta"]), 1e-3)
                check_penalty(g[lo:hi], og, f"nbins={nbins} seg {s}")
            assert largest > 12288 and (clamped > 0 or nbins == 20000), (largest, clamped, [int(f) for f in rrec["flags"]], [float(a) for a in frec["alpha"]])   # the case reaches past every set of private bins


def test_quantize_rate_segmented_with_histograms(gg):
    sizes = [0, 17, 4096, 1, 30_000, 0, 99_999, 16384]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    x = make(int(off[-1]), 0.02, 0.7, seed=8)
    delta_h = np.array([0.01, 0.002, 0.0, 0.004, 0.001, 0.01, float("nan"), 0.0005], dtype=np.float32)
    delta = torch.tensor(delta_h, device=DEV)
    ws = gg.Workspace(x.numel(), len(sizes))
    out, hist, sym = gg.gg_quantize_rate_segmented(x, off, delta, ws, eg_k=0, nbins=512, want_symbols=True)
    rec = gg.rate_records(out)
    hist = hist.cpu().numpy().view(np.uint64).reshape(len(sizes), 512)
    sym = sym.cpu().numpy()
    hb = host_bits(x)
    for s, sz in enumerate(sizes):
        d = delta_h[s]
        if sz == 0:
            assert rec[s]["flags"] == gg.GG_F_EMPTY and rec[s]["eg_bits"] == 0 and rec[s]["fl_bits"] == 1
            continue
        if not (d > 0 and np.isfinite(d)):
            assert rec[s]["flags"] == gg.GG_F_DEGENERATE and rec[s]["eg_bits"] == 0
            assert not sym[off[s]:off[s + 1]].any() and not hist[s].any()
            continue
        r, ohist, osym = oracle.quantize_rate(hb[off[s]:off[s + 1]], float(d), nbins=512, want_symbols=True)
        check_rate(rec[s], r, f"seg {s}")
        assert np.array_equal(hist[s], ohist) and np.array_equal(sym[off[s]:off[s + 1]], osym)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_histogram_sweep_layouts_and_transitions(gg, dtype):
    """The histogram-only sweep counts in one of two LDS layouts, chosen per piece from the data (copies of the low
    bins for peaked symbol distributions, plain bins otherwise).  A bucket of 6 M elements -- more chunks than the
    sweep has workgroups, so that a workgroup walks through several units -- whose units alternate between peaked
    and wide distributions, with NaN / Inf / zeros planted, tiny, empty and degenerate units in between: every
    count, bit sum, largest symbol and flag against the oracle, for histograms narrower and wider than either
    layout, both rounding modes, two code orders."""
    rng = np.random.default_rng(5)
    sizes, kinds = [], []
    for i in range(60):
        sizes.append(int(rng.choice([0, 1, 777, 5000, 16384, 40_001, 131_072, 300_000])))
        kinds.append(i % 3)
    sizes += [1_200_000, 900_001]
    kinds += [0, 1]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n, S = int(off[-1]), len(sizes)
    assert n > 256 * 16384
    x = torch.empty(n, dtype=torch.float32, device=DEV)
    delta_h = np.empty(S, dtype=np.float32)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(55)
    for s in range(S):
        lo, hi = int(off[s]), int(off[s + 1])
        if kinds[s] == 0:       # peaked: nearly every symbol below a thousand
            x[lo:hi] = gg_inputs.gg_torch(hi - lo, 0.02, 0.8, gen, DEV)
            delta_h[s] = 0.02 / 8
        elif kinds[s] == 1:     # wide: symbols in the thousands and tens of thousands
            x[lo:hi] = gg_inputs.gg_torch(hi - lo, 0.5, 1.6, gen, DEV)
            delta_h[s] = 0.5 / 3000
        else:                   # in between, with a heavy tail
            x[lo:hi] = gg_inputs.gg_torch(hi - lo, 1e-3, 0.5, gen, DEV)
            delta_h[s] = 1e-3 / 16
    delta_h[7] = 0.0                                   # a unit without a usable step
    pos = torch.randint(0, n, (400,), generator=gen, device=DEV)
    x[pos[:100]] = float("nan")
    x[pos[100:200]] = float("inf")
    x[pos[200:300]] = -float("inf")
    x[pos[300:]] = 0.0
    x = x.to(dtype)
    hb = host_bits(x)
    delta = torch.tensor(delta_h, device=DEV)
    ws = gg.Workspace(n, S)
    for nbins, mode, k in ((2, gg.GG_FLOOR, 0), (40, gg.GG_NEAREST_EVEN, 0), (1024, gg.GG_FLOOR, 3), (1500, gg.GG_FLOOR, 0),
                           (4096, gg.GG_NEAREST_EVEN, 1), (40000, gg.GG_FLOOR, 0), (65536, gg.GG_FLOOR, 0)):
        out, hist, _ = gg.gg_quantize_rate_segmented(x, off, delta, ws, eg_k=k, round_mode=mode, nbins=nbins)
        rec = gg.rate_records(out)
        hist = hist.cpu().numpy().view(np.uint64).reshape(S, nbins)

        def one(s):
            return oracle.quantize_rate(hb[off[s]:off[s + 1]], float(delta_h[s]), eg_k=k, round_mode=mode, nbins=nbins)

        live = [s for s in range(S) if sizes[s] > 0 and delta_h[s] > 0]
        for s, (r, ohist, _) in zip(live, parity.oracle_threads(one, live)):
            check_rate(rec[s], r, f"nbins {nbins} unit {s} kind {kinds[s]}")
            assert np.array_equal(hist[s], ohist), (nbins, s)
        assert rec[7]["flags"] == gg.GG_F_DEGENERATE and not hist[7].any()
        for s in range(S):
            if sizes[s] == 0:
                assert rec[s]["flags"] == gg.GG_F_EMPTY and not hist[s].any()
    # the same through the single-tensor call: one unit shared by every workgroup
    out, hist1, _ = gg.gg_quantize_rate(x, 0.02 / 8, ws, nbins=4096)
    r, ohist, _ = oracle.quantize_rate(hb, 0.02 / 8, nbins=4096)
    check_rate(gg.rate_records(out)[0], r, "whole buffer")
    assert np.array_equal(hist1.cpu().numpy().view(np.uint64), ohist)


def test_quantize_rate_rows(gg):
    rows, cols = 37, 4096
    x = make(rows * cols, 0.5, 0.8, seed=4, dtype=torch.bfloat16)
    ws = gg.Workspace(rows * cols, rows)
    fit = gg.gg_fit_rows(x, rows, cols, ws)
    delta = gg.gg_delta_from_fit(fit, rows, 8.0)
    frec = gg.fit_records(fit)
    dh = delta.cpu().numpy()
    assert np.array_equal(dh, frec["alpha"] / np.float32(8.0))
    out, _ = gg.gg_quantize_rate_rows(x, rows, cols, delta, ws)
    rec = gg.rate_records(out)
    hb = host_bits(x)
    for r_ in range(rows):
        r, _, _ = oracle.quantize_rate(hb[r_ * cols:(r_ + 1) * cols], float(dh[r_]))
        check_rate(rec[r_], r, f"row {r_}", entropy=False)


# ---- penalty ------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("beta", [0.5, 0.8, 1.0, 1.5, 2.0, 3.0])
def test_penalty_grad(gg, beta, dtype):
    n = 100_003
    alpha, lam = 0.015, 1e-4
    w = make(n, alpha, beta, seed=int(beta * 10), dtype=dtype)
    w[::1000] = 0.0
    g = gg.gg_penalty_grad(w, alpha, beta, lam)
    og = oracle.penalty_grad(host_bits(w), alpha, beta, lam)
    check_penalty(g.cpu().numpy(), og, f"beta={beta}")
    assert not g.cpu().numpy()[::1000].any()
    base = torch.randn(n, device=DEV)
    acc = gg.gg_penalty_grad(w, alpha, beta, lam, grad=base.clone(), accumulate=True)
    oacc = oracle.penalty_grad(host_bits(w), alpha, beta, lam, grad=base.cpu().numpy().copy(), accumulate=True)
    check_penalty(acc.cpu().numpy(), oacc, f"acc beta={beta}", penalty=og)


def test_penalty_segmented_uses_fitted_parameters(gg):
    segs = gg_inputs.scaled_layout(gg_inputs.weights_7b()[:18], 3001)
    segs.insert(3, gg_inputs.Segment("zeros", 50))
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=4, device=DEV, dtype=torch.bfloat16, alpha_range=(0.005, 0.03),
                                            beta_range=(0.6, 2.0), log_alpha=False)
    flat[int(off[3]):int(off[4])] = 0
    ws = gg.Workspace(flat.numel(), len(segs))
    fit = gg.gg_fit_segmented(flat, off, ws)
    frec = gg.fit_records(fit)
    grad = gg.gg_penalty_grad_segmented(flat, off, fit, 1e-4, ws).cpu().numpy()
    hb = host_bits(flat)
    for s in range(len(segs)):
        lo, hi = int(off[s]), int(off[s + 1])
        if frec[s]["alpha"] == 0:
            assert not grad[lo:hi].any()
            continue
        og = oracle.penalty_grad(hb[lo:hi], frec[s]["alpha"], frec[s]["beta"], 1e-4)
        check_penalty(grad[lo:hi], og, segs[s].name)


# ---- sampler ------------------------------------------------------------------------------------
def test_philox_words_bit_exact(gg):
    for seed, stream, offset, attempt in [(0, 0, 0, 0), (0xDEADBEEFCAFEF00D, 7, (1 << 32) - 3, 2), (5, 0xFFFFFFFF, 1 << 40, 63)]:
        w = gg.gg_philox_words(64, seed, stream, offset, attempt).cpu().numpy().view(np.uint32).reshape(64, 4)
        for i in (0, 1, 2, 3, 31, 63):
            idx = offset + i
            exp = oracle.philox4x32_10([attempt, stream, idx & 0xFFFFFFFF, idx >> 32], [seed & 0xFFFFFFFF, seed >> 32])
            assert list(map(int, w[i])) == exp


@pytest.mark.parametrize("alpha,beta", [(0.02, 1.0), (0.015, 1.5), (0.5, 0.8), (1e-4, 0.5), (0.01, 2.0), (1.0, 0.1),
                                        (2.0, 6.0), (0.3, 0.05), (0.3, 20.0)])      # the last two: the ends of the shape range
def test_sample_tracks_oracle_and_distribution(gg, alpha, beta):
    from scipy import stats
    n = 200_000
    x = gg.gg_sample(n, alpha, beta, seed=42, stream_id=3, offset=12345).cpu().numpy()
    o = oracle.sample(n, alpha, beta, seed=42, stream=3, offset=12345)
    # same generator words, fp32 vs fp64 transcendentals: nearly every element agrees closely; the rest
    # (an accept/reject decision that flipped on a rounding difference) must still be valid draws
    close = np.abs(x - o) <= 2e-4 * np.abs(o) + 1e-30
    assert close.mean() > 0.999, close.mean()
    assert np.array_equal(np.sign(x), np.sign(o))
    a32 = float(np.float32(alpha))
    assert stats.kstest((np.abs(x.astype(np.float64)) / a32) ** beta, "gamma", args=(1.0 / beta,)).pvalue > 1e-3
    # launch-shape independence: a sub-range drawn separately is identical
    y = gg.gg_sample(1000, alpha, beta, seed=42, stream_id=3, offset=12345 + 777).cpu().numpy()
    assert np.array_equal(y, x[777:1777])


def test_sample_bf16_and_fit_round_trip(gg):
    n = 1 << 21
    a = gg.gg_init_alpha(4096, 0.7, 2.0)
    x = gg.gg_sample(n, a, 0.7, seed=9, dtype=torch.bfloat16)
    xf = gg.gg_sample(n, a, 0.7, seed=9, dtype=torch.float32)
    assert torch.equal(x, xf.to(torch.bfloat16))
    ws = gg.Workspace(n, 1)
    rec = gg.fit_records(gg.gg_fit(xf, ws))[0]
    assert abs(float(rec["beta"]) - 0.7) < 0.02
    # Eq. 5: variance xi / d_in
    assert float(rec["sum_sq"]) / n == pytest.approx(2.0 / 4096, rel=0.02)


# ---- the whole pass over a bucket ---------------------------------------------------------------
@pytest.mark.parametrize("dtype,mode,k", [(torch.float32, 0, 0), (torch.bfloat16, 1, 2)])
def test_fused_segmented_small_bucket(gg, dtype, mode, k):
    layout = gg_inputs.gradient_bucket_1p5b()
    segs = gg_inputs.scaled_layout(layout[:18] + layout[-1:], 499)
    segs.insert(2, gg_inputs.Segment("empty", 0))
    segs.insert(7, gg_inputs.Segment("zeros", 33))
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=3, device=DEV, dtype=dtype)
    flat[int(off[7]):int(off[8])] = 0
    S = len(segs)
    ws = gg.Workspace(flat.numel(), S)
    grad0 = torch.randn(flat.numel(), device=DEV)
    res = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, eg_k=k, round_mode=mode, nbins=2048, want_symbols=True,
                                lam=1e-4, grad=grad0.clone(), accumulate=True)
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    hist = res["hist"].cpu().numpy().view(np.uint64).reshape(S, 2048)
    sym = res["symbols"].cpu().numpy()
    grad = res["grad"].cpu().numpy()
    hb = host_bits(flat)
    g0 = grad0.cpu().numpy()
    for s in range(S):
        lo, hi = int(off[s]), int(off[s + 1])
        of = oracle.fit(hb[lo:hi])
        check_fit(frec[s], of, segs[s].name)
        # the step is one fp32 division of the GPU's own alpha
        assert np.float32(rrec[s]["delta"]) == np.float32(frec[s]["alpha"]) / np.float32(16.0)
        if hi == lo:
            assert rrec[s]["flags"] == gg.GG_F_EMPTY
            continue
        if frec[s]["alpha"] == 0:
            assert rrec[s]["flags"] == gg.GG_F_DEGENERATE and rrec[s]["eg_bits"] == 0 and rrec[s]["fl_bits"] == 0
            assert np.array_equal(grad[lo:hi], g0[lo:hi])
            continue
        r, ohist, osym = oracle.quantize_rate(hb[lo:hi], float(rrec[s]["delta"]), eg_k=k, round_mode=mode, nbins=2048,
                                              want_symbols=True)
        check_rate(rrec[s], r, segs[s].name)
        assert np.array_equal(hist[s], ohist) and np.array_equal(sym[lo:hi], osym)
        og = oracle.penalty_grad(hb[lo:hi], frec[s]["alpha"], frec[s]["beta"], 1e-4, grad=g0[lo:hi].copy(),
                                 accumulate=True)
        check_penalty(grad[lo:hi], og, segs[s].name,
                      penalty=oracle.penalty_grad(hb[lo:hi], frec[s]["alpha"], frec[s]["beta"], 1e-4))


def test_fused_matches_oracle_fused_and_is_reproducible(gg):
    layout = gg_inputs.gradient_bucket_1p5b()
    segs = gg_inputs.scaled_layout(layout[:27], 211)
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=13, device=DEV)
    S = len(segs)
    ws = gg.Workspace(flat.numel(), S)
    res = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0)
    res2 = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0)
    assert res["fit"].cpu().numpy().tobytes() == res2["fit"].cpu().numpy().tobytes()
    assert res["rate"].cpu().numpy().tobytes() == res2["rate"].cpu().numpy().tobytes()
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    # oracle's own whole pass, fed the GPU's steps (same bits) so the integer results must be identical
    fits, rates = oracle.fused_segmented(host_bits(flat), off, delta_div=0.0, delta=rrec["delta"].copy())
    for s in range(S):
        check_fit(frec[s], fits[s], segs[s].name)
        check_rate(rrec[s], rates[s], segs[s].name, entropy=False)
        # and the GPU's step agrees with the oracle's own alpha/16 to the parameter tolerance
        assert float(rrec[s]["delta"]) == pytest.approx(float(np.float32(fits[s].alpha) / np.float32(16)), rel=1e-4)


def test_fused_rows_activation_like(gg):
    rows, cols = 96, 4096
    x = gg_inputs.make_tensor((rows, cols), 0.5, 0.8, seed=2, device=DEV, dtype=torch.bfloat16, outlier_frac=1e-3,
                              outlier_scale=20.0).reshape(-1)
    ws = gg.Workspace(rows * cols, rows)
    res = gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, want_total=True)
    frec, rrec, tot = gg.fit_records(res["fit"]), gg.rate_records(res["rate"]), gg.fit_records(res["total"])[0]
    hb = host_bits(x)
    check_fit(tot, oracle.fit(hb), "total")
    for r_ in range(rows):
        xs = hb[r_ * cols:(r_ + 1) * cols]
        check_fit(frec[r_], oracle.fit(xs), f"row {r_}")
        r, _, _ = oracle.quantize_rate(xs, float(rrec[r_]["delta"]))
        check_rate(rrec[r_], r, f"row {r_}", entropy=False)
    # per-tensor histogram + entropy with the step from the total fit
    delta = float(np.float32(tot["alpha"]) / np.float32(8.0))
    out, hist, _ = gg.gg_quantize_rate(x, delta, ws, nbins=32768)
    r, ohist, _ = oracle.quantize_rate(hb, delta, nbins=32768)
    check_rate(gg.rate_records(out)[0], r, "tensor")
    assert np.array_equal(hist.cpu().numpy().view(np.uint64), ohist)


@pytest.mark.parametrize("dtype,cols", [(torch.bfloat16, 100), (torch.float32, 67)])
def test_fused_rows_taken_two_at_a_time(gg, dtype, cols):
    """Matrices of many short rows: a wave takes two rows per turn and one lane per row solves the fit.
    The odd row count leaves a last turn with a single row; the row length is no multiple of a vector."""
    rows = 16387
    x = make(rows * cols, 0.3, 1.2, seed=31, dtype=dtype)
    # a constant row (no usable step) and a zero row in the middle of pairs
    x.view(rows, cols)[5] = 0.25
    x.view(rows, cols)[8] = 0.0
    ws = gg.Workspace(rows * cols, rows)
    grad = torch.zeros(rows * cols, device=DEV)
    res = gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, lam=1e-3, grad=grad, want_symbols=True)
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    sym, g = res["symbols"].cpu().numpy(), res["grad"].cpu().numpy()
    hb = host_bits(x)
    picks = sorted(set([0, 1, 2, 3, 4, 5, 6, 7, 8, 9, rows - 3, rows - 2, rows - 1]) | set(range(11, rows, 997)))
    for r_ in picks:
        xs = hb[r_ * cols:(r_ + 1) * cols]
        check_fit(frec[r_], oracle.fit(xs), f"row {r_}")
        if r_ == 8:
            assert int(rrec[r_]["flags"]) & gg.GG_F_DEGENERATE
            continue
        r, _, osym = oracle.quantize_rate(xs, float(rrec[r_]["delta"]), want_symbols=True)
        check_rate(rrec[r_], r, f"row {r_}", entropy=False)
        assert np.array_equal(sym[r_ * cols:(r_ + 1) * cols], osym)
        check_penalty(g[r_ * cols:(r_ + 1) * cols], oracle.penalty_grad(xs, frec[r_]["alpha"], frec[r_]["beta"], 1e-3), f"row {r_}")
    # every row, against the sums the records themselves must satisfy
    assert np.all(frec["n"] == cols)
    assert int(rrec["n"].astype(np.int64).sum()) == rows * cols


@pytest.mark.parametrize("dtype,cols", [(torch.bfloat16, 4096), (torch.bfloat16, 8), (torch.bfloat16, 520), (torch.bfloat16, 1544),
                                        (torch.bfloat16, 3592), (torch.float32, 2048), (torch.float32, 4), (torch.float32, 772),
                                        (torch.float32, 1284)])
@pytest.mark.parametrize("mode", ["floor", "nearest"])
def test_fused_rows_kept_in_registers(gg, dtype, cols, mode):
    """Rows of at most 8 KiB made of whole 16-byte vectors, fit + order-0 rate: the wave keeps the row in registers
    between its two sweeps, 1 to 8 vectors per lane, the last group of 64 vectors full or short, and fits the row
    with the fp32-based solver.  Shapes from 0.06 to 19 along the rows; rows holding NaN, Inf, zeros, one value."""
    rows = 1100
    rng = np.random.default_rng(cols)
    betas = np.exp(rng.uniform(np.log(0.06), np.log(19.0), size=rows))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(cols)
    x = torch.empty(rows, cols, device=DEV)
    for lo in range(0, rows, 50):          # a shape per group of 50 rows
        x[lo:lo + 50] = gg_inputs.gg_torch(min(50, rows - lo) * cols, 0.3, float(betas[lo]), gen, DEV).reshape(-1, cols)
    x[3] = 0.0
    x[4] = -0.75
    x[5, cols // 2] = float("nan")
    x[6, 0] = float("inf")
    x[7, cols - 1] = -float("inf")
    x[8] *= 1e-30
    x = x.to(dtype).reshape(-1)
    rmode = gg.GG_FLOOR if mode == "floor" else gg.GG_NEAREST_EVEN
    ws = gg.Workspace(rows * cols, rows)
    res = gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, round_mode=rmode, want_total=True)
    frec, rrec, tot = gg.fit_records(res["fit"]), gg.rate_records(res["rate"]), gg.fit_records(res["total"])[0]
    hb = host_bits(x)

    def one(r_):
        xs = hb[r_ * cols:(r_ + 1) * cols]
        d = float(rrec[r_]["delta"])
        return oracle.fit(xs), (oracle.quantize_rate(xs, d, round_mode=rmode)[0] if d > 0 and np.isfinite(d) else None)

    for r_, (f, r) in enumerate(parity.oracle_threads(one, range(rows))):
        check_fit(frec[r_], f, f"row {r_} beta {betas[r_ - r_ % 50]:.3f}")
        if r is None:
            assert int(rrec[r_]["flags"]) & gg.GG_F_DEGENERATE, r_
        else:
            check_rate(rrec[r_], r, f"row {r_}", entropy=False)
            assert rrec[r_]["delta"] == np.float32(frec[r_]["alpha"]) / np.float32(8.0)
    assert int(rrec[5]["flags"]) & gg.GG_F_NONFINITE or int(rrec[5]["flags"]) & gg.GG_F_DEGENERATE
    if not (np.isnan(tot["sum_abs"]) or np.isinf(tot["sum_abs"])):
        check_fit(tot, oracle.fit(hb), "whole matrix")
    else:
        assert int(tot["flags"]) & gg.GG_F_NONFINITE
    # the same rows through the general wave-per-row kernel (symbols asked for): the records have to agree
    res2 = gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, round_mode=rmode, want_symbols=True)
    f2, r2 = gg.fit_records(res2["fit"]), gg.rate_records(res2["rate"])
    for r_ in range(0, rows, 37):
        if rrec[r_]["delta"] == r2[r_]["delta"]:
            for k in ("eg_bits", "u_max", "fl_bits", "flags"):
                assert rrec[r_][k] == r2[r_][k], (r_, k)
        assert abs(float(frec[r_]["beta"]) - float(f2[r_]["beta"])) <= 2e-5 * float(f2[r_]["beta"]), r_


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fit_at_very_small_and_very_large_scales(gg, dtype):
    """Eq. 3 has no range condition: tensors whose squares underflow or overflow fp32 (values around 1e-25 and 1e25,
    down to fp32 denormals) are fitted like any other -- every entry point that sums moments, against the oracle."""
    n = 150_001
    base = make(n, 1.0, 0.9, seed=77).float()
    hb_of = lambda t: host_bits(t)
    ws = gg.Workspace(4 * n, 4)
    for scale in (1e-25, 1e25, 3e-36, 2e37):
        x = (base * scale).to(dtype)
        o = oracle.fit(hb_of(x))
        assert o.flags == 0 and abs(o.beta - 0.9) < 0.05
        check_fit(gg.fit_records(gg.gg_fit(x, ws))[0], o, f"tensor x {scale}")
    # a bucket that mixes the scales (each unit its own), with an ordinary unit between them; the fused one-sweep mode too
    parts = [base * 1e-25, base[:40_000], base * 1e25, base[:7] * 1e-30]
    flat = torch.cat(parts).to(dtype)
    off = np.concatenate([[0], np.cumsum([p_.numel() for p_ in parts])]).astype(np.int64)
    hb = hb_of(flat)
    rec = gg.fit_records(gg.gg_fit_segmented(flat, off, ws))
    for s_ in range(4):
        check_fit(rec[s_], oracle.fit(hb[off[s_]:off[s_ + 1]]), f"unit {s_}")
    res = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0)
    rec2, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    delta = res["rate"].new_empty(0)
    for s_ in range(4):
        check_fit(rec2[s_], oracle.fit(hb[off[s_]:off[s_ + 1]]), f"fused unit {s_}")
        r, _, _ = oracle.quantize_rate(hb[off[s_]:off[s_ + 1]], float(rrec[s_]["delta"]))
        check_rate(rrec[s_], r, f"fused unit {s_}", entropy=False)
    steps = gg.gg_delta_from_fit(res["fit"], 4, 16.0)
    res1 = gg.gg_fused_segmented(flat, off, ws, delta_div=0.0, delta=steps)          # moments and rate from one sweep
    rec3 = gg.fit_records(res1["fit"])
    for s_ in range(4):
        check_fit(rec3[s_], oracle.fit(hb[off[s_]:off[s_ + 1]]), f"one-sweep unit {s_}")
    # rows: the general wave-per-row kernel (symbols asked for) and the one that keeps rows in registers
    rows, cols = 300, 512
    m = (make(rows * cols, 1.0, 1.3, seed=78).float().reshape(rows, cols) *
         torch.logspace(-30, 30, rows, device=DEV).reshape(rows, 1)).to(dtype).reshape(-1)
    hm = hb_of(m)
    wsr = gg.Workspace(rows * cols, rows)
    for kw in (dict(want_symbols=True), dict()):
        fr = gg.fit_records(gg.gg_fused_rows(m, rows, cols, wsr, delta_div=8.0, **kw)["fit"])
        for r_ in range(rows):
            check_fit(fr[r_], oracle.fit(hm[r_ * cols:(r_ + 1) * cols]), f"row {r_} {kw}")
    fr = gg.fit_records(gg.gg_fit_rows(m, rows, cols, wsr))
    for r_ in range(rows):
        check_fit(fr[r_], oracle.fit(hm[r_ * cols:(r_ + 1) * cols]), f"fit_rows {r_}")


def test_fit_only_and_penalty_only_fused_modes(gg):
    segs = gg_inputs.scaled_layout(gg_inputs.weights_7b()[:9], 2003)
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=4, device=DEV, dtype=torch.bfloat16, alpha_range=(0.005, 0.03),
                                            beta_range=(0.6, 2.0), log_alpha=False)
    S = len(segs)
    ws = gg.Workspace(flat.numel(), S)
    grad = torch.zeros(flat.numel(), device=DEV)
    res = gg.gg_fused_segmented(flat, off, ws, want_rate=False, lam=1e-4, grad=grad, accumulate=False)
    assert res["rate"] is None
    frec = gg.fit_records(res["fit"])
    hb = host_bits(flat)
    g = res["grad"].cpu().numpy()
    for s in range(S):
        lo, hi = int(off[s]), int(off[s + 1])
        check_fit(frec[s], oracle.fit(hb[lo:hi]), segs[s].name)
        check_penalty(g[lo:hi], oracle.penalty_grad(hb[lo:hi], frec[s]["alpha"], frec[s]["beta"], 1e-4), segs[s].name)


def test_many_small_units_use_the_per_lane_solver(gg):
    """More than 2048 units switch the finalisation to one lane per unit; results must not change."""
    rng = np.random.default_rng(5)
    sizes = rng.integers(0, 400, size=3000)
    sizes[17] = 40_000                      # one unit spanning several chunks among the small ones
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    gen = torch.Generator(device=DEV)
    gen.manual_seed(21)
    x = torch.empty(n, device=DEV)
    betas = rng.uniform(0.4, 3.0, size=sizes.size)
    for s in range(0, sizes.size, 100):     # a shape per group of 100 units
        lo, hi = int(off[s]), int(off[min(s + 100, sizes.size)])
        x[lo:hi] = gg_inputs.gg_torch(hi - lo, 0.01, float(betas[s]), gen, DEV)
    ws = gg.Workspace(n, sizes.size)
    res = gg.gg_fused_segmented(x, off, ws, delta_div=16.0)
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    hb = host_bits(x)
    fits, rates = oracle.fused_segmented(hb, off, delta_div=0.0, delta=rrec["delta"].copy())
    for s in range(sizes.size):
        check_fit(frec[s], fits[s], f"unit {s}")
        if frec[s]["alpha"] > 0:
            check_rate(rrec[s], rates[s], f"unit {s}", entropy=False)
    # rows path with the same switch
    rows, cols = 2500, 96
    xr = make(rows * cols, 0.5, 0.8, seed=3, dtype=torch.bfloat16)
    wsr = gg.Workspace(rows * cols, rows)
    rec = gg.fit_records(gg.gg_fit_rows(xr, rows, cols, wsr))
    hbr = host_bits(xr)
    for r_ in range(0, rows, 7):
        check_fit(rec[r_], oracle.fit(hbr[r_ * cols:(r_ + 1) * cols]), f"row {r_}")


def test_fused_pass_is_graph_capturable(gg):
    """The library enqueues kernels only (tables travel as kernel arguments; no allocation, memset,
    copy or synchronisation), so a whole pass can be captured into a HIP graph and replayed."""
    segs = gg_inputs.scaled_layout(gg_inputs.gradient_bucket_1p5b()[:27], 211)
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=17, device=DEV)
    S = len(segs)
    ws = gg.Workspace(flat.numel(), S)
    fit = torch.empty(S * 40, dtype=torch.uint8, device=DEV)
    rate = torch.empty(S * 48, dtype=torch.uint8, device=DEV)
    grad = torch.empty(flat.numel(), device=DEV)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, lam=1e-4, grad=grad, fit=fit, rate=rate)   # warm-up
    torch.cuda.current_stream().wait_stream(stream)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, lam=1e-4, grad=grad, fit=fit, rate=rate)
    for rep in range(3):
        flat.mul_(1.0 + 0.25 * rep)              # eager work between replays, new input values
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (fit.cpu().numpy().tobytes(), rate.cpu().numpy().tobytes(), grad.cpu().numpy().tobytes())
        e_fit = torch.empty_like(fit)
        e_rate = torch.empty_like(rate)
        e_grad = torch.empty_like(grad)
        gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, lam=1e-4, grad=e_grad, fit=e_fit, rate=e_rate)
        torch.cuda.synchronize()
        assert got == (e_fit.cpu().numpy().tobytes(), e_rate.cpu().numpy().tobytes(), e_grad.cpu().numpy().tobytes()), rep


@pytest.mark.parametrize("seed", range(48))
def test_random_buckets_and_options_against_the_oracle(gg, seed):
    """Seeded random unit layouts (empty, tiny, sizes around the chunk of 16384 elements, a few large) with
    random dtype, rounding, order k, bins, symbols and penalty mode: every unit against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    S = int(rng.integers(1, 40))
    kinds = rng.integers(0, 6, size=S)
    sizes = np.where(kinds == 0, 0,
            np.where(kinds == 1, rng.integers(1, 9, size=S),
            np.where(kinds == 2, 16384 * rng.integers(1, 4, size=S) + rng.integers(-2, 3, size=S),
            np.where(kinds == 3, rng.integers(9, 5000, size=S),
            np.where(kinds == 4, rng.integers(5000, 70_000, size=S), 4 * rng.integers(1, 2000, size=S))))))
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    dtype = torch.bfloat16 if rng.integers(2) else torch.float32
    mode = int(rng.integers(2))
    k = int(rng.choice([0, 0, 1, 2, 5]))
    nbins = int(rng.choice([0, 2, 64, 1000, 20000]))
    want_symbols = bool(rng.integers(2))
    lam = float(rng.choice([0.0, 1e-4]))
    accumulate = bool(rng.integers(2))
    div = float(rng.choice([4.0, 16.0, 64.0]))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(2000 + seed)
    parts = [gg_inputs.gg_torch(int(sz), float(10.0 ** rng.uniform(-4, 0)), float(rng.uniform(0.4, 2.5)), gen, DEV, dtype)
             for sz in sizes]
    flat = torch.cat(parts) if n else torch.empty(0, device=DEV, dtype=dtype)
    if n and S > 2 and sizes[1] > 0:
        flat[int(off[1]):int(off[2])] = 0                   # a unit of zeros: no step, no penalty
    if S > 4 and sizes[3] > 0:
        flat[int(off[3]) + int(sizes[3]) // 2] = float("nan")   # moments not finite: no fit, no step
    if S > 5 and sizes[4] > 1:
        flat[int(off[4]) + 1] = float("-inf")
    g0 = (torch.randn(n, device=DEV, generator=gen) * 1e-3) if lam > 0 else None
    grad = g0.clone() if lam > 0 else None
    ws = gg.Workspace(n, S)
    res = gg.gg_fused_segmented(flat, off, ws, delta_div=div, eg_k=k, round_mode=mode, nbins=nbins,
                                want_symbols=want_symbols, lam=lam, grad=grad, accumulate=accumulate)
    torch.cuda.synchronize()
    what = f"seed {seed}: S={S} n={n} {dtype} mode={mode} k={k} nbins={nbins} sym={want_symbols} lam={lam} acc={accumulate}"
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    hb = host_bits(flat)
    hist = res["hist"].cpu().numpy().view(np.uint64).reshape(S, nbins) if nbins else None
    sym = res["symbols"].cpu().numpy() if want_symbols else None
    gout = grad.cpu().numpy() if lam > 0 else None
    g0h = g0.cpu().numpy() if lam > 0 else None
    for u in range(S):
        lo, hi = int(off[u]), int(off[u + 1])
        xs = hb[lo:hi]
        where = f"{what}, unit {u} [{lo}, {hi})"
        check_fit(frec[u], oracle.fit(xs), where)
        if hi == lo:
            assert int(rrec[u]["flags"]) & gg.GG_F_EMPTY and int(rrec[u]["eg_bits"]) == 0, where
            continue
        if float(frec[u]["alpha"]) == 0.0:
            assert int(rrec[u]["flags"]) == gg.GG_F_DEGENERATE and int(rrec[u]["eg_bits"]) == 0, where
            if lam > 0:
                assert np.array_equal(gout[lo:hi], g0h[lo:hi] if accumulate else np.zeros(hi - lo, np.float32)), where
            continue
        r, ohist, osym = oracle.quantize_rate(xs, float(rrec[u]["delta"]), eg_k=k, round_mode=mode, nbins=nbins,
                                              want_symbols=want_symbols)
        check_rate(rrec[u], r, where, entropy=nbins > 0)
        if nbins:
            assert np.array_equal(hist[u], ohist), where
        if want_symbols:
            assert np.array_equal(sym[lo:hi], osym), where
        if lam > 0:
            bare = oracle.penalty_grad(xs, frec[u]["alpha"], frec[u]["beta"], lam)
            if accumulate:
                og = oracle.penalty_grad(xs, frec[u]["alpha"], frec[u]["beta"], lam, grad=g0h[lo:hi].copy(), accumulate=True)
                check_penalty(gout[lo:hi], og, where, penalty=bare)
            else:
                check_penalty(gout[lo:hi], bare, where)


@pytest.mark.parametrize("seed", range(16))
def test_random_matrices_by_rows_against_the_oracle(gg, seed):
    """Seeded random row-shaped inputs (short rows taken by a wave, long rows cut into chunks; with and without
    symbols, penalty, given steps): sampled rows against the oracle, the whole-matrix fit against all of it."""
    rng = np.random.default_rng(3000 + seed)
    cols = int(rng.choice([1, 7, 64, 100, 1000, 4096, 16384, 16385, 40_000]))
    rows = int(rng.integers(1, max(2, min(3000, 600_000 // cols))))
    dtype = torch.bfloat16 if rng.integers(2) else torch.float32
    mode = int(rng.integers(2))
    k = int(rng.choice([0, 0, 3]))
    want_symbols = bool(rng.integers(2))
    lam = float(rng.choice([0.0, 1e-3]))
    given = bool(rng.integers(3) == 0)                      # steps handed in instead of alpha / div
    x = make(rows * cols, float(10.0 ** rng.uniform(-3, 0)), float(rng.uniform(0.5, 2.2)), seed=4000 + seed, dtype=dtype)
    if rows > 3:
        x[cols * 1 + cols // 2] = float("nan")              # row 1: moments not finite
        x[cols * 2] = float("inf")                          # row 2 likewise
    steps = (torch.rand(rows, device=DEV) * 0.05 + 1e-3) if given else None
    grad = torch.zeros(rows * cols, device=DEV) if lam > 0 else None
    ws = gg.Workspace(rows * cols, rows)
    res = gg.gg_fused_rows(x, rows, cols, ws, delta_div=0.0 if given else 8.0, delta=steps, eg_k=k, round_mode=mode,
                           want_symbols=want_symbols, lam=lam, grad=grad, want_total=True)
    torch.cuda.synchronize()
    what = f"seed {seed}: {rows}x{cols} {dtype} mode={mode} k={k} sym={want_symbols} lam={lam} given={given}"
    frec, rrec, tot = gg.fit_records(res["fit"]), gg.rate_records(res["rate"]), gg.fit_records(res["total"])[0]
    hb = host_bits(x)
    check_fit(tot, oracle.fit(hb), what + ", total")
    sym = res["symbols"].cpu().numpy() if want_symbols else None
    g = grad.cpu().numpy() if lam > 0 else None
    for r_ in sorted(set(rng.integers(0, rows, size=min(rows, 12)).tolist()) | {0, rows - 1} | set(range(min(rows, 4)))):
        xs = hb[r_ * cols:(r_ + 1) * cols]
        where = f"{what}, row {r_}"
        check_fit(frec[r_], oracle.fit(xs), where)
        if not given and float(frec[r_]["alpha"]) == 0.0:   # no fit (zeros, NaN, Inf): no step, nothing coded, no penalty
            assert int(rrec[r_]["flags"]) == gg.GG_F_DEGENERATE and int(rrec[r_]["eg_bits"]) == 0, where
            if lam > 0:
                assert not g[r_ * cols:(r_ + 1) * cols].any(), where
            continue
        if given:
            assert float(rrec[r_]["delta"]) == float(steps[r_]), where
        r, _, osym = oracle.quantize_rate(xs, float(rrec[r_]["delta"]), eg_k=k, round_mode=mode, want_symbols=want_symbols)
        check_rate(rrec[r_], r, where, entropy=False)
        if want_symbols:
            assert np.array_equal(sym[r_ * cols:(r_ + 1) * cols], osym), where
        if lam > 0:
            check_penalty(g[r_ * cols:(r_ + 1) * cols], oracle.penalty_grad(xs, frec[r_]["alpha"], frec[r_]["beta"], lam), where)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_one_unit_bucket_with_and_without_a_unit_table(gg, dtype):
    """A bucket of one unit starting at element 0 is handled as a plain tensor (no unit table); the same
    unit behind 16 other elements goes through the table.  Same data, same chunks: the same records."""
    n, pad = 250_007, 16
    x = make(n, 0.01, 0.7, seed=88, dtype=dtype)
    padded = torch.cat([torch.ones(pad, device=DEV, dtype=dtype), x])
    ws, wsp = gg.Workspace(n, 1), gg.Workspace(n + pad, 1)
    grad, gradp = torch.zeros(n, device=DEV), torch.zeros(n + pad, device=DEV)
    a = gg.gg_fused_segmented(x, [0, n], ws, delta_div=16.0, nbins=1024, want_symbols=True, lam=1e-4, grad=grad)
    b = gg.gg_fused_segmented(padded, [pad, pad + n], wsp, delta_div=16.0, nbins=1024, want_symbols=True, lam=1e-4, grad=gradp)
    torch.cuda.synchronize()
    for key in ("fit", "rate", "hist"):
        assert a[key].cpu().numpy().tobytes() == b[key].cpu().numpy().tobytes(), key
    assert torch.equal(a["symbols"], b["symbols"][pad:]) and torch.equal(grad, gradp[pad:])
    frec, rrec = gg.fit_records(a["fit"]), gg.rate_records(a["rate"])
    hb = host_bits(x)
    check_fit(frec[0], oracle.fit(hb), "one unit")
    r, ohist, osym = oracle.quantize_rate(hb, float(rrec[0]["delta"]), nbins=1024, want_symbols=True)
    check_rate(rrec[0], r, "one unit")
    assert np.array_equal(a["hist"].cpu().numpy().view(np.uint64), ohist) and np.array_equal(a["symbols"].cpu().numpy(), osym)


def test_two_streams_with_their_own_workspaces_do_not_interfere(gg):
    """The library keeps no state between calls: passes over different buffers, enqueued on two streams
    (default priority) so that they overlap, give what each gives alone."""
    segs = gg_inputs.scaled_layout(gg_inputs.gradient_bucket_1p5b()[:40], 53)
    jobs = []
    for seed in (41, 42):
        flat, off, _, _ = gg_inputs.make_bucket(segs, seed=seed, device=DEV)
        ws = gg.Workspace(flat.numel(), len(segs))
        alone = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, nbins=512)
        torch.cuda.synchronize()
        jobs.append((flat, off, ws, [alone[k].cpu().numpy().tobytes() for k in ("fit", "rate", "hist")]))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    outs = [None, None]
    for rep in range(4):                                   # interleaved submission
        for i, (flat, off, ws, _) in enumerate(jobs):
            with torch.cuda.stream(streams[i]):
                outs[i] = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0, nbins=512)
    torch.cuda.synchronize()
    for i, (_, _, _, alone) in enumerate(jobs):
        assert [outs[i][k].cpu().numpy().tobytes() for k in ("fit", "rate", "hist")] == alone, i


def test_rows_histogram_coder_and_sampler_are_graph_capturable(gg):
    """The other launch paths under capture: the wave-per-row pass and the block-private histogram (both ask the
    runtime for occupancy figures while launching), the coder in both directions, the sampler.  Replays with
    eager work between them have to give what eager calls give on the same inputs."""
    rows, cols = 300, 512
    n = rows * cols
    x = make(n, 0.3, 1.1, seed=9, dtype=torch.bfloat16)
    ws, ws1 = gg.Workspace(n, rows), gg.Workspace(n, 1)
    bufs = gg.eg_buffers(n, None, DEV)
    tiles = (n + gg.GG_EG_TILE - 1) // gg.GG_EG_TILE

    def work():
        r = gg.gg_fused_rows(x, rows, cols, ws, delta_div=8.0, want_total=True)
        rate, hist, sym = gg.gg_quantize_rate(x, 0.01, ws1, nbins=4096, want_symbols=True)
        rate_h, hist_h, _ = gg.gg_quantize_rate(x, 0.01, ws1, nbins=2048)          # the histogram-only sweep
        gg.gg_eg_encode_tensor(x, 0.01, buffers=bufs)
        back = gg.gg_eg_decode_dequant(bufs[0], bufs[1][: tiles + 1], n, 0.01)
        smp = gg.gg_sample(5000, 0.1, 0.7, seed=3)
        return [r["fit"], r["rate"], r["total"], rate, hist, sym, rate_h, hist_h, bufs[2], back, smp]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work()                                             # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        outs = work()
    for rep in range(3):
        x.mul_(1.0 + 0.5 * rep)                            # eager work between replays, new input values
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.cpu().numpy().tobytes() for t in outs]
        want = [t.cpu().numpy().tobytes() for t in work()]
        torch.cuda.synchronize()
        assert got == want, rep


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fused_one_sweep_mode_with_given_steps(gg, dtype):
    """Steps handed in (no dependence on this call's fit): moments and rate from one read of x."""
    layout = gg_inputs.gradient_bucket_1p5b()
    segs = gg_inputs.scaled_layout(layout[:18] + layout[-1:], 311)
    segs.insert(3, gg_inputs.Segment("empty", 0))
    flat, off, alpha, _ = gg_inputs.make_bucket(segs, seed=23, device=DEV, dtype=dtype)
    S = len(segs)
    ws = gg.Workspace(flat.numel(), S)
    dh = (np.insert(alpha, 3, 1e-4) / 16.0).astype(np.float32)          # "previous step's" steps
    dh[5] = 0.0                                                          # one unit without a usable step
    delta = torch.tensor(dh, device=DEV)
    res = gg.gg_fused_segmented(flat, off, ws, delta_div=0.0, delta=delta, nbins=1024, want_symbols=True)
    frec, rrec = gg.fit_records(res["fit"]), gg.rate_records(res["rate"])
    hist = res["hist"].cpu().numpy().view(np.uint64).reshape(S, 1024)
    sym = res["symbols"].cpu().numpy()
    hb = host_bits(flat)
    for s in range(S):
        lo, hi = int(off[s]), int(off[s + 1])
        check_fit(frec[s], oracle.fit(hb[lo:hi]), segs[s].name)
        assert np.float32(rrec[s]["delta"]) == dh[s]
        if hi == lo:
            assert rrec[s]["flags"] == gg.GG_F_EMPTY
            continue
        if not dh[s] > 0:
            assert rrec[s]["flags"] == gg.GG_F_DEGENERATE and rrec[s]["eg_bits"] == 0
            continue
        r, ohist, osym = oracle.quantize_rate(hb[lo:hi], float(dh[s]), nbins=1024, want_symbols=True)
        check_rate(rrec[s], r, segs[s].name)
        assert np.array_equal(hist[s], ohist) and np.array_equal(sym[lo:hi], osym)
    # without histogram / symbols (the lean kernel) the integers are the same
    res2 = gg.gg_fused_segmented(flat, off, ws, delta_div=0.0, delta=delta)
    r2 = gg.rate_records(res2["rate"])
    assert np.array_equal(r2["eg_bits"], rrec["eg_bits"]) and np.array_equal(r2["u_max"], rrec["u_max"])
    f2 = gg.fit_records(res2["fit"])
    assert np.allclose(f2["sum_sq"], frec["sum_sq"], rtol=1e-12) and np.allclose(f2["beta"], frec["beta"], rtol=1e-6)
