"""GPU parity of the pass's companions in the training algorithms (rate gradient, GCT update,
Exp-Golomb bit stream) against the oracle."""
import numpy as np
import pytest
import torch

import gg_inputs
import oracle
from parity import host_bits

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


def inv32(delta):
    return float(np.float32(1.0) / np.float32(delta))


# ---- rate gradient ------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,k", [(1, 0), (4099, 0), (100_003, 2), (16384 * 3 + 5, 1)])
def test_rate_grad(gg, n, k, dtype):
    x = make(n, 0.5, 0.8, seed=n, dtype=dtype)
    x[::97] = 0.0
    delta = 2.0 ** -6
    g = gg.gg_rate_grad(x, delta, eg_k=k, scale=0.37).cpu().numpy()
    o = oracle.rate_grad(host_bits(x), inv32(delta), k, n, scale=0.37)
    # fp32 coefficient and one fp32 division against the oracle's fp64: a few 1e-7 relative
    assert np.allclose(g, o, rtol=1e-5, atol=1e-30)
    assert not g[::97].any()
    base = torch.randn(n, device=DEV)
    acc = gg.gg_rate_grad(x, delta, eg_k=k, scale=0.37, grad=base.clone(), accumulate=True).cpu().numpy()
    assert np.allclose(acc, base.cpu().numpy() + o, rtol=1e-6, atol=1e-5 * np.abs(o).max())


def test_rate_grad_matches_gct_rate_term(gg):
    # with ghat_prev = 2g and eps = 0, h = 1/(2 eta): ghat - g = lambda * dR/dg / (2 eta)
    n = 50_000
    g = make(n, 1e-3, 1.0, seed=3)
    g[g == 0] = 1e-3
    w = torch.zeros(n, device=DEV)
    gp = (2 * g).clone()
    delta = 2.0 ** -14
    gg.gg_gct_update(w, g, gp, eta=0.5, lam=1.0, eps=0.0, delta=delta, eg_k=0)
    dr = gg.gg_rate_grad(g, delta, eg_k=0)
    assert torch.allclose(gp - g, dr, rtol=1e-4, atol=1e-7 * float(dr.abs().max()))


# ---- GCT update ---------------------------------------------------------------------------------
def gct_case(n, seed):
    g = make(n, 1e-3, 0.9, seed=seed)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed + 100)
    gp = g * (1.0 + 0.5 * torch.randn(n, device=DEV, generator=gen))   # previous equivalent gradient near g
    w = torch.randn(n, device=DEV, generator=gen)
    return w, g, gp


def check_gct(w_gpu, gp_gpu, w0, g, gp0, eta, lam, eps, delta, k, n_rate, first):
    wo, go, gpo = w0.copy(), g.copy(), gp0.copy()
    oracle.gct_update(wo, go, gpo, eta, lam, eps, inv32(delta), k, n_rate, first)
    # conditioning: the secant term (1 - g/(ghat_prev+eps))/eta carries an absolute fp32 error of
    # ~2^-23 max(1, |g/(ghat_prev+eps)|)/eta, multiplied by lambda*|dR/dg| in the equivalent gradient
    dr = np.abs(oracle.rate_grad(g, inv32(delta), k, n_rate).astype(np.float64))
    ratio = np.abs(g.astype(np.float64) / (gp0.astype(np.float64) + eps))
    tol_g = 1e-6 * np.abs(gpo) + (0 if first else 4e-7 * abs(lam) * dr / eta * np.maximum(1.0, ratio)) + 1e-30
    assert np.all(np.abs(gp_gpu.astype(np.float64) - gpo) <= tol_g), float(np.max(np.abs(gp_gpu - gpo) / tol_g))
    tol_w = 2.0 ** -23 * np.abs(wo) + eta * tol_g
    assert np.all(np.abs(w_gpu.astype(np.float64) - wo) <= tol_w)


@pytest.mark.parametrize("n", [1, 5, 4099, 16384 * 2 + 3, 300_001])
@pytest.mark.parametrize("first", [True, False])
def test_gct_update_single(gg, n, first):
    w, g, gp = gct_case(n, seed=n)
    w0, g0, gp0 = w.cpu().numpy(), g.cpu().numpy(), gp.cpu().numpy()
    eta, lam, eps, delta, k = 1e-2, 0.3, 1e-8, 2.0 ** -16, 0
    gg.gg_gct_update(w, g, gp, eta, lam, eps, delta, eg_k=k, first_step=first)
    check_gct(w.cpu().numpy(), gp.cpu().numpy(), w0, g0, gp0, eta, lam, eps, delta, k, n, first)
    if first:   # t = 1: plain SGD, the equivalent gradient is the gradient itself
        assert np.array_equal(gp.cpu().numpy(), g0)


def test_gct_zero_lambda_is_sgd(gg):
    w, g, gp = gct_case(100_000, seed=9)
    w0, g0 = w.cpu().numpy(), g.cpu().numpy()
    gg.gg_gct_update(w, g, gp, 1e-2, 0.0, 1e-8, 2.0 ** -16)
    assert np.array_equal(gp.cpu().numpy(), g0)
    expect = (w0.astype(np.float64) - float(np.float32(1e-2)) * g0.astype(np.float64))
    assert np.all(np.abs(w.cpu().numpy() - expect) <= 2.0 ** -23 * np.abs(expect))


def test_gct_update_segmented_with_fitted_steps(gg):
    layout = gg_inputs.gradient_bucket_1p5b()
    segs = gg_inputs.scaled_layout(layout[:18], 499)
    segs.insert(4, gg_inputs.Segment("empty", 0))
    segs.insert(9, gg_inputs.Segment("zeros", 40))
    g, off, _, _ = gg_inputs.make_bucket(segs, seed=3, device=DEV)
    g[int(off[9]):int(off[10])] = 0
    n, S = g.numel(), len(segs)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1)
    gp = g * (1.0 + 0.5 * torch.randn(n, device=DEV, generator=gen))
    gp[int(off[9]):int(off[10])] = 1e-3
    w = torch.randn(n, device=DEV, generator=gen)
    ws = gg.Workspace(n, S)
    res = gg.gg_fused_segmented(g, off, ws, delta_div=16.0)           # the pass gives each tensor's step
    rrec = gg.rate_records(res["rate"])
    delta = torch.tensor(rrec["delta"].copy(), device=DEV)
    w0, g0, gp0 = w.cpu().numpy(), g.cpu().numpy(), gp.cpu().numpy()
    eta, lam, eps = 1e-2, 0.2, 1e-8
    gg.gg_gct_update_segmented(w, g, gp, off, delta, eta, lam, eps, ws)
    wg, gpg = w.cpu().numpy(), gp.cpu().numpy()
    for s in range(S):
        lo, hi = int(off[s]), int(off[s + 1])
        if hi == lo:
            continue
        d = float(rrec["delta"][s])
        if not d > 0:     # no usable step: plain SGD
            assert np.array_equal(gpg[lo:hi], g0[lo:hi])
            continue
        check_gct(wg[lo:hi], gpg[lo:hi], w0[lo:hi], g0[lo:hi], gp0[lo:hi], eta, lam, eps, d, 0, hi - lo, False)


# ---- Exp-Golomb bit stream ----------------------------------------------------------------------
@pytest.mark.parametrize("n", [0, 1, 7, 2047, 2048, 2049, 100_003])
@pytest.mark.parametrize("k", [0, 3])
def test_eg_stream_equals_oracle_stream(gg, n, k):
    x = make(max(n, 1), 0.02, 0.7, seed=n + k)[:n].contiguous()
    ws = gg.Workspace(max(n, 1), 1)
    delta = float(np.float32(0.02) / np.float32(16))
    out, _, sym = gg.gg_quantize_rate(x, delta, ws, eg_k=k, want_symbols=True) if n else (None, None,
                                                                                         torch.empty(0, dtype=torch.int32, device=DEV))
    stream, index, total = gg.gg_eg_encode(sym, eg_k=k)
    q = sym.cpu().numpy()
    u = np.where(q > 0, 2 * q.astype(np.int64) - 1, -2 * q.astype(np.int64)).astype(np.uint32)
    obuf, obits = oracle.eg_encode(u, k)
    assert total == obits
    if n:
        assert total == int(gg.rate_records(out)[0]["eg_bits"])       # the rate estimate is the stream size
    sb = stream.cpu().numpy()
    assert np.array_equal(sb[: obuf.size], obuf)
    assert not sb[obuf.size: (obuf.size + 3) // 4 * 4].any()      # the last word is zero-padded
    idx = index.cpu().numpy()
    assert idx[0] == 0 and idx[-1] == total and np.all(np.diff(idx) >= 0)
    back = gg.gg_eg_decode(stream, index, n, eg_k=k)
    assert np.array_equal(back.cpu().numpy(), q)
    # the oracle decodes the GPU stream too
    assert np.array_equal(oracle.eg_decode(sb, total, k, n), u)


def test_eg_stream_extreme_symbols_and_tight_capacity(gg):
    q = torch.tensor([0, 1, -1, 2 ** 30, -(2 ** 30), 5, -7, 0, 0, 123456, -654321] * 400, dtype=torch.int32, device=DEV)
    for k in (0, 15):
        u = np.array([oracle.map_symbol(int(v)) for v in q.cpu().numpy()], dtype=np.uint32)
        obuf, obits = oracle.eg_encode(u, k)
        stream, index, total = gg.gg_eg_encode(q, eg_k=k, capacity_bytes=(obits + 7) // 8)
        assert total == obits
        assert np.array_equal(stream.cpu().numpy()[: obuf.size], obuf)
        assert np.array_equal(gg.gg_eg_decode(stream, index, q.numel(), eg_k=k).cpu().numpy(), q.cpu().numpy())
    # a stream that is too small: the total still reports the need, nothing is written past the end
    stream, index, total = gg.gg_eg_encode(q, eg_k=0, capacity_bytes=64)
    assert total == oracle.eg_encode(np.array([oracle.map_symbol(int(v)) for v in q.cpu().numpy()], dtype=np.uint32), 0)[1]
    assert total > 64 * 8 and stream.numel() == 64


def test_eg_decode_of_bytes_that_are_no_code_stream(gg):
    # What the decoder reads and writes does not depend on what the stream holds: under the index of a real stream,
    # bytes that are no code stream (random, all zero = endless prefixes, all one = shortest codes) decode to
    # something, the call returns, and nothing but the n outputs is written.
    n = 70 * gg.GG_EG_TILE + 19
    rng = np.random.default_rng(11)
    q = torch.tensor(rng.integers(-300, 301, size=n).astype(np.int32), device=DEV)
    for k in (0, 3):
        stream, index, total = gg.gg_eg_encode(q, eg_k=k)
        fills = [torch.tensor(rng.integers(0, 256, size=stream.numel()).astype(np.uint8), device=DEV),
                 torch.zeros_like(stream), torch.full_like(stream, 0xFF)]
        for other in fills:
            buf = torch.full((n + 256,), 12345, dtype=torch.int32, device=DEV)
            gg.gg_eg_decode(other, index, n, eg_k=k, out=buf[:n])
            fbuf = torch.full((n + 256,), 7.0, dtype=torch.float32, device=DEV)
            gg.gg_eg_decode_dequant(other, index, n, 0.5, eg_k=k, out=fbuf[:n], accumulate=True)
            torch.cuda.synchronize()
            assert bool((buf[n:] == 12345).all()) and bool((fbuf[n:] == 7.0).all())
        # with k = 0 a one bit is the whole code of u = 0, so all-one bytes decode to zeros from a tile's first bit on
        if k == 0:
            ones = gg.gg_eg_decode(fills[2], index, n, eg_k=0)
            assert bool((ones[: gg.GG_EG_TILE] == 0).all())
        assert torch.equal(gg.gg_eg_decode(stream, index, n, eg_k=k), q)     # and the real stream still decodes


def test_eg_stream_truncated_by_capacity(gg):
    # the stream buffer ends inside the data: every packing tile (2048 symbols) that fits is written whole,
    # wherever the cut falls relative to the groups of four tiles a workgroup packs
    n = 11 * 2048 + 77
    rng = np.random.default_rng(5)
    qh = rng.integers(-40, 41, size=n).astype(np.int32)
    qh[rng.integers(0, n, size=50)] = rng.integers(-2 ** 20, 2 ** 20, size=50).astype(np.int32)
    q = torch.tensor(qh, device=DEV)
    u = np.where(qh > 0, 2 * qh.astype(np.int64) - 1, -2 * qh.astype(np.int64)).astype(np.uint32)
    for k in (0, 2):
        obuf, obits = oracle.eg_encode(u, k)
        lens = 2 * np.floor(np.log2(u.astype(np.float64) + float(1 << k))).astype(np.int64) - k + 1
        tile_end = np.cumsum(lens)[np.minimum(np.arange(1, 13) * 2048, n) - 1]      # bit offset after each tile
        assert tile_end[-1] == obits
        for cut in range(1, 12):
            for slack in (0, 4, 8):        # capacity just at / beyond the end of tile `cut`
                cap = (int(tile_end[cut - 1]) + 31) // 32 * 4 + slack
                stream, index, total = gg.gg_eg_encode(q, eg_k=k, capacity_bytes=cap)
                assert total == obits and stream.numel() == cap
                fit = int(np.searchsorted(tile_end, cap * 8, side="right"))            # tiles that end within the buffer
                assert fit >= cut
                good_bits = int(tile_end[fit - 1])
                sb = stream.cpu().numpy()
                whole = good_bits // 8
                assert np.array_equal(sb[:whole], obuf[:whole]), (k, cut, slack)
                if good_bits % 8:
                    mask = (0xFF << (8 - good_bits % 8)) & 0xFF
                    assert (sb[whole] & mask) == (obuf[whole] & mask)
                # the index does not depend on the buffer
                idx = index.cpu().numpy()
                assert np.array_equal(idx[1:-1], np.cumsum(lens)[gg.GG_EG_TILE - 1::gg.GG_EG_TILE][: idx.size - 2])


@pytest.mark.parametrize("k", [1, 7, 15])
def test_eg_stream_orders_and_tile_multiples(gg, k):
    rng = np.random.default_rng(k)
    for n in (256, 2048 - 256, 4 * 2048, 8 * 2048 + 255, 8 * 2048 + 256 + 1):
        qh = (rng.standard_cauchy(n) * 30).clip(-2 ** 29, 2 ** 29).astype(np.int32)
        q = torch.tensor(qh, device=DEV)
        u = np.where(qh > 0, 2 * qh.astype(np.int64) - 1, -2 * qh.astype(np.int64)).astype(np.uint32)
        obuf, obits = oracle.eg_encode(u, k)
        stream, index, total = gg.gg_eg_encode(q, eg_k=k)
        assert total == obits
        assert np.array_equal(stream.cpu().numpy()[: obuf.size], obuf)
        assert torch.equal(gg.gg_eg_decode(stream, index, n, eg_k=k), q)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("mode", [0, 1])
def test_eg_stream_straight_from_the_tensor(gg, dtype, mode):
    # quantise + encode in one call == rate sweep's symbols through the coder == the oracle's stream
    n = 3 * 8192 + 2048 + 333
    x = make(n, 0.02, 0.7, seed=31, dtype=dtype)
    special = torch.tensor([float("nan"), float("inf"), -float("inf"), 1e30, -1e30, 0.0, -0.0, 1e-30, -1e-30, 0.00124999, -0.00125],
                           device=DEV).to(dtype)
    x[100:100 + special.numel()] = special
    x[-special.numel():] = special
    delta = float(np.float32(0.02) / np.float32(16))
    ws = gg.Workspace(n, 1)
    for k in (0, 2):
        out, _, sym = gg.gg_quantize_rate(x, delta, ws, eg_k=k, round_mode=mode, want_symbols=True)
        s_ref, i_ref, t_ref = gg.gg_eg_encode(sym, eg_k=k)
        s_new, i_new, t_new = gg.gg_eg_encode_tensor(x, delta, eg_k=k, round_mode=mode)
        assert t_new == t_ref == int(gg.rate_records(out)[0]["eg_bits"])
        nbytes = (t_ref + 7) // 8
        assert torch.equal(s_new[:nbytes], s_ref[:nbytes]) and torch.equal(i_new, i_ref)
        r, _, osym = oracle.quantize_rate(host_bits(x), delta, eg_k=k, round_mode=mode, want_symbols=True)
        u = np.where(osym > 0, 2 * osym.astype(np.int64) - 1, -2 * osym.astype(np.int64)).astype(np.uint32)
        obuf, obits = oracle.eg_encode(u, k)
        assert t_new == obits == r.eg_bits
        assert np.array_equal(s_new.cpu().numpy()[: obuf.size], obuf)
        assert torch.equal(gg.gg_eg_decode(s_new, i_new, n, eg_k=k), sym)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_eg_stream_of_a_bucket_with_a_step_per_unit(gg, dtype):
    # unit boundaries inside tiles, inside a lane's eight symbols, empty / one-element / unusable-step units
    sizes = [0, 17, 4096, 1, 30_000, 0, 99_999, 16_384, 3, 1, 1, 5, 3 * 2048 + 5, 0, 2048, 7]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(off[-1])
    x = make(n, 0.02, 0.7, seed=41, dtype=dtype)
    delta_h = np.array([0.01, 0.002, 0.0, 0.004, 0.001, 0.01, float("nan"), 0.0005, 0.003, 0.02, 0.001, 0.004, 0.0007,
                        0.1, 0.0011, 0.05], dtype=np.float32)
    delta = torch.tensor(delta_h, device=DEV)
    ws = gg.Workspace(n, len(sizes))
    hb = host_bits(x)
    for mode, k in ((0, 0), (1, 3)):
        out, _, sym = gg.gg_quantize_rate_segmented(x, off, delta, ws, eg_k=k, round_mode=mode, want_symbols=True)
        s_ref, i_ref, t_ref = gg.gg_eg_encode(sym, eg_k=k)
        s_new, i_new, t_new = gg.gg_eg_encode_segmented(x, off, delta, ws, eg_k=k, round_mode=mode)
        assert t_new == t_ref
        nbytes = (t_ref + 7) // 8
        assert torch.equal(s_new[:nbytes], s_ref[:nbytes]) and torch.equal(i_new, i_ref)
        # the oracle's symbols unit by unit (an unusable step gives zeros), then its stream
        osym = np.zeros(n, dtype=np.int32)
        bits = 0
        rec = gg.rate_records(out)
        for u, sz in enumerate(sizes):
            d = delta_h[u]
            if sz == 0 or not (d > 0 and np.isfinite(d)):
                bits += sz * (k + 1)                    # symbol 0 costs k + 1 bits
                continue
            r, _, q = oracle.quantize_rate(hb[off[u]:off[u + 1]], float(d), eg_k=k, round_mode=mode, want_symbols=True)
            osym[off[u]:off[u + 1]] = q
            bits += r.eg_bits
            assert int(rec[u]["eg_bits"]) == r.eg_bits
        uu = np.where(osym > 0, 2 * osym.astype(np.int64) - 1, -2 * osym.astype(np.int64)).astype(np.uint32)
        obuf, obits = oracle.eg_encode(uu, k)
        assert t_new == obits == bits
        assert np.array_equal(s_new.cpu().numpy()[: obuf.size], obuf)
        assert np.array_equal(gg.gg_eg_decode(s_new, i_new, n, eg_k=k).cpu().numpy(), osym)


def test_bucket_round_trip_reconstructs_within_one_step(gg):
    # fit -> steps -> one stream for the bucket -> decode -> q * Delta: the floor quantiser leaves 0 <= x - q Delta < Delta
    # (up to the fp32 rounding of x / Delta), and the stream is as long as the pass said
    segs = gg_inputs.scaled_layout(gg_inputs.gradient_bucket_1p5b()[:19], 211)
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=9, device=DEV)
    n, S = flat.numel(), len(segs)
    ws = gg.Workspace(n, S)
    res = gg.gg_fused_segmented(flat, off, ws, delta_div=16.0)
    rrec = gg.rate_records(res["rate"])
    delta = gg.gg_delta_from_fit(res["fit"], S, 16.0)
    stream, index, total = gg.gg_eg_encode_segmented(flat, off, delta, ws)
    assert total == int(rrec["eg_bits"].astype(np.uint64).sum())
    q = gg.gg_eg_decode(stream, index, n)
    per_elem = torch.repeat_interleave(delta, torch.tensor(np.diff(off), device=DEV))
    err = flat.double() - q.double() * per_elem.double()
    tol = 4e-7 * flat.abs().double()                      # x * (1/Delta) is rounded twice in fp32
    assert bool((err >= -tol).all()) and bool((err < per_elem.double() + tol).all())
    assert float(total) / n < 32.0                        # and it does compress an fp32 gradient


@pytest.mark.parametrize("n,k", [(1, 0), (255, 0), (4099, 1), (300_001, 0), (1 << 20, 3)])
def test_eg_stream_decoded_straight_to_values(gg, n, k):
    """Decode + reconstruct in one kernel: q * delta per element, written or added to what is there."""
    x = make(n, 0.02, 0.9, seed=60 + k)
    delta = 0.02 / 16
    stream, index, total = gg.gg_eg_encode_tensor(x, delta, eg_k=k)
    hb = host_bits(x)
    _, _, q = oracle.quantize_rate(hb, delta, eg_k=k, want_symbols=True)
    want = oracle.dequantize(q, delta)
    got = gg.gg_eg_decode_dequant(stream, index, n, delta, eg_k=k)
    assert np.array_equal(got.cpu().numpy(), want)
    base = torch.linspace(-1, 1, n, device=DEV)
    acc = gg.gg_eg_decode_dequant(stream, index, n, delta, eg_k=k, out=base.clone(), accumulate=True)
    assert np.array_equal(acc.cpu().numpy(), oracle.dequantize(q, delta, out=base.cpu().numpy().copy(), accumulate=True))
    # and it agrees with decoding to symbols first
    sym = gg.gg_eg_decode(stream, index, n, eg_k=k)
    assert np.array_equal(sym.cpu().numpy(), q)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_bucket_stream_decoded_straight_to_values_with_a_step_per_unit(gg, dtype):
    """Bucket -> one stream -> values: every element comes back as q * (its unit's step), bit for bit what the
    oracle's symbols and steps give; units of zeros (no step) come back as zeros; accumulate adds."""
    sizes = [5000, 0, 3, 1, 40_000, 0, 0, 257, 16384, 2, 70_001, 255]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    S, n = len(sizes), int(off[-1])
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    flat = torch.cat([gg_inputs.gg_torch(sz, 10.0 ** (-1 - (i % 3)), 0.6 + 0.15 * i, gen, DEV, dtype) for i, sz in enumerate(sizes)])
    flat[int(off[7]):int(off[8])] = 0                      # a unit of zeros: its fit gives no step
    ws = gg.Workspace(n, S)
    fit = gg.gg_fit_segmented(flat, off, ws)
    steps = gg.gg_delta_from_fit(fit, S, 16.0)
    stream, index, total = gg.gg_eg_encode_segmented(flat, off, steps, ws, eg_k=1)
    got = gg.gg_eg_decode_dequant_segmented(stream, index, off, steps, ws, eg_k=1).cpu().numpy()
    base = torch.linspace(-2, 2, n, device=DEV)
    acc = gg.gg_eg_decode_dequant_segmented(stream, index, off, steps, ws, eg_k=1, out=base.clone(), accumulate=True).cpu().numpy()
    hb, st, b0 = host_bits(flat), steps.cpu().numpy(), base.cpu().numpy()
    for u in range(S):
        lo, hi = int(off[u]), int(off[u + 1])
        if hi == lo:
            continue
        if not (st[u] > 0 and np.isfinite(st[u])):
            assert u == 7 and not got[lo:hi].any() and np.array_equal(acc[lo:hi], b0[lo:hi])
            continue
        _, _, q = oracle.quantize_rate(hb[lo:hi], float(st[u]), eg_k=1, want_symbols=True)
        assert np.array_equal(got[lo:hi], oracle.dequantize(q, float(st[u]))), u
        assert np.array_equal(acc[lo:hi], oracle.dequantize(q, float(st[u]), out=b0[lo:hi].copy(), accumulate=True)), u
        x = hb[lo:hi] if dtype == torch.float32 else gg_inputs.bf16_bits_to_f32(hb[lo:hi])
        assert np.all(np.abs(x - got[lo:hi]) <= st[u] * (1 + 1e-5))       # within one step of the input


def test_eg_stream_of_longest_codes(gg):
    # every symbol takes 63 bits (k = 0): the decoder's buffered words run out within a step and are topped up
    n = 5000
    q = torch.full((n,), 2 ** 30, dtype=torch.int32, device=DEV)
    q[1::2] = -(2 ** 30)
    u = np.array([oracle.map_symbol(int(v)) for v in q.cpu().numpy()], dtype=np.uint32)
    obuf, obits = oracle.eg_encode(u, 0)
    stream, index, total = gg.gg_eg_encode(q, eg_k=0)
    assert total == obits
    assert np.array_equal(stream.cpu().numpy()[: obuf.size], obuf)
    assert torch.equal(gg.gg_eg_decode(stream, index, n, eg_k=0), q)


def test_eg_stream_many_tiles(gg):
    # more packing tiles (2048 symbols) than one scan group holds (8192), ragged last tile
    n = 2 * 8192 * 2048 + 12345
    x = make(n, 0.02, 0.9, seed=21)
    ws = gg.Workspace(n, 1)
    out, _, sym = gg.gg_quantize_rate(x, 0.02 / 16.0, ws, want_symbols=True)
    stream, index, total = gg.gg_eg_encode(sym, eg_k=0)
    assert total == int(gg.rate_records(out)[0]["eg_bits"])
    q = sym.cpu().numpy()
    u = np.where(q > 0, 2 * q.astype(np.int64) - 1, -2 * q.astype(np.int64)).astype(np.uint32)
    obuf, obits = oracle.eg_encode(u, 0)
    assert total == obits
    assert np.array_equal(stream.cpu().numpy()[: obuf.size], obuf)
    idx = index.cpu().numpy()
    assert idx.size == (n + gg.GG_EG_TILE - 1) // gg.GG_EG_TILE + 1 and idx[0] == 0 and idx[-1] == total
    # index entries are the bit offsets of every GG_EG_TILE-th symbol
    lens = 2 * np.floor(np.log2(u.astype(np.float64) + 1.0)).astype(np.int64) + 1
    assert np.array_equal(idx[1:-1], np.cumsum(lens)[gg.GG_EG_TILE - 1::gg.GG_EG_TILE][: idx.size - 2])
    assert torch.equal(gg.gg_eg_decode(stream, index, n, eg_k=0), sym)


# ---- torch glue: GG init driver, differentiable rate, GCT state ---------------------------------
def test_gg_init_driver(gg):
    w1 = torch.empty(512, 1024, device=DEV)                       # fan-in 1024
    w2 = torch.empty(2048, 256, device=DEV, dtype=torch.bfloat16)  # fan-in 256
    gg.gg_init_([(w1, 1024), (w2, 256)], shape=0.5, xi=2.0, seed=7)
    assert float(w1.double().var()) == pytest.approx(2.0 / 1024, rel=0.05)   # Eq. 5: variance xi / fan_in
    assert float(w2.double().var()) == pytest.approx(2.0 / 256, rel=0.05)
    rec = gg.fit_records(gg.gg_fit(w1.view(-1), gg.Workspace(w1.numel(), 1)))[0]
    assert abs(float(rec["beta"]) - 0.5) < 0.02
    a1 = gg.gg_init_alpha(1024, 0.5, 2.0)
    ref = gg.gg_sample(w1.numel(), a1, 0.5, 7, stream_id=0)
    assert torch.equal(ref, w1.view(-1))                           # tensor i = generator stream i


def test_differentiable_eg_rate(gg):
    a = make(40_000, 0.5, 0.8, seed=1).reshape(100, 400).requires_grad_(True)
    delta = 2.0 ** -5
    r = gg.eg_rate(a, delta, 0)
    ws = gg.Workspace(a.numel(), 1)
    rec = gg.rate_records(gg.gg_quantize_rate(a.detach().view(-1), delta, ws)[0])[0]
    assert float(r.detach()) == pytest.approx(float(rec["eg_bits"]) / a.numel(), rel=1e-6)
    (3.0 * r).backward()
    o = oracle.rate_grad(host_bits(a.detach().view(-1)), inv32(delta), 0, a.numel(), scale=3.0)
    assert np.allclose(a.grad.view(-1).cpu().numpy(), o, rtol=1e-5, atol=1e-30)


def test_gct_state_runs_algorithm_2_steps(gg):
    segs = gg_inputs.scaled_layout(gg_inputs.gradient_bucket_1p5b()[:9], 997)
    off = gg_inputs.offsets_of(segs)
    n = int(off[-1])
    st = gg.GCTState(n, off, eta=1e-2, lam=0.1, decay=0.8)
    w = torch.randn(n, device=DEV)
    base, _, _, _ = gg_inputs.make_bucket(segs, seed=50, device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    for t in range(3):
        g = base * (1.0 + 0.2 * torch.randn(n, device=DEV, generator=gen))    # slowly varying gradient
        w0, gp0 = w.cpu().numpy().copy(), st.ghat_prev.cpu().numpy().copy()   # state before the step
        res = st.step(w, g)
        rrec = gg.rate_records(res["rate"])
        g_h, w1, gp1 = g.cpu().numpy(), w.cpu().numpy(), st.ghat_prev.cpu().numpy()
        for s in range(len(segs)):            # oracle: the same update per tensor with the GPU's step
            lo, hi = int(off[s]), int(off[s + 1])
            check_gct(w1[lo:hi], gp1[lo:hi], w0[lo:hi], g_h[lo:hi], gp0[lo:hi], 1e-2, st.lam, 1e-8,
                      float(rrec["delta"][s]), 0, hi - lo, t == 0)
    st.end_epoch()
    assert st.lam == pytest.approx(0.08) and st.t == 4
