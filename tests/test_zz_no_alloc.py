"""The entry point that allocates nothing (gg_fused_segmented_noalloc: the pass with the library's own scratch
array) against gg_fused_segmented with a caller's workspace: same kernels, so every output byte must agree --
on two calls in a row, the second on a smaller bucket (the array keeps what the first call left in it)."""
import ctypes as C

import numpy as np
import pytest
import torch

import gg_inputs
import paper_2506_00486_amd as gg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(flat, off, nbins, want_symbols, lam, accumulate, eg_k=0, delta_div=16.0):
    """Runs the workspace call and the no-allocation call on the same inputs; returns the two sets of output bytes."""
    S, n = len(off) - 1, flat.numel()
    ws = gg.Workspace(int(off[-1]), S, device=DEV)
    g0 = torch.randn(n, device=DEV) if lam else None
    ga = g0.clone() if lam else None
    ref = gg.gg_fused_segmented(flat, off, ws, delta_div=delta_div, eg_k=eg_k, nbins=nbins, want_symbols=want_symbols,
                                lam=lam, grad=ga, accumulate=accumulate)
    fit = torch.empty(max(S, 1) * 40, dtype=torch.uint8, device=DEV)
    rate = torch.empty(max(S, 1) * 48, dtype=torch.uint8, device=DEV)
    hist = torch.empty(max(S, 1) * nbins, dtype=torch.int64, device=DEV) if nbins else None
    sym = torch.empty(n, dtype=torch.int32, device=DEV) if want_symbols else None
    gb = g0.clone() if lam else None
    gg.gg_fused_segmented_noalloc(flat, off, fit, rate, delta_div=delta_div, eg_k=eg_k, nbins=nbins, hist=hist, symbols=sym,
                                  lam=lam, grad=gb, accumulate=accumulate)
    torch.cuda.synchronize()
    a = dict(fit=ref["fit"], rate=ref["rate"], hist=ref["hist"], symbols=ref["symbols"], grad=ga)
    b = dict(fit=fit, rate=rate, hist=hist, symbols=sym, grad=gb)
    return a, b


def _same(a, b, where):
    for k in a:
        if a[k] is None:
            assert b[k] is None, (where, k)
            continue
        equal = a[k].cpu().numpy().tobytes() == b[k].cpu().numpy().tobytes()   # outside the assert: no byte diff on failure
        assert equal, (where, k)


def test_noalloc_matches_workspace_call_twice_second_smaller():
    # first: a ragged bucket of a few hundred thousand elements (several chunks per unit, shared runs, an empty unit)
    segs = [gg_inputs.Segment("a", 300_001), gg_inputs.Segment("b", 0), gg_inputs.Segment("c", 1537),
            gg_inputs.Segment("d", 131_072), gg_inputs.Segment("e", 70_003)]
    flat, off, _, _ = gg_inputs.make_bucket(segs, seed=11, device=DEV)
    a, b = _both(flat, off, nbins=4096, want_symbols=True, lam=1e-4, accumulate=True)
    _same(a, b, "first call")
    frec = gg.fit_records(b["fit"])
    assert int(frec["n"].sum()) == flat.numel() and (frec["flags"][1] & gg.GG_F_EMPTY)
    # second: smaller, other layout and options, bf16 -- whatever the first call left in the array must not show
    segs2 = [gg_inputs.Segment("p", 20_000), gg_inputs.Segment("q", 777)]
    flat2, off2, _, _ = gg_inputs.make_bucket(segs2, seed=12, device=DEV, dtype=torch.bfloat16)
    a2, b2 = _both(flat2, off2, nbins=0, want_symbols=False, lam=0.0, accumulate=False, eg_k=2, delta_div=8.0)
    _same(a2, b2, "second call")
    # and the first bucket again: the result is a function of the inputs alone
    a3, b3 = _both(flat, off, nbins=4096, want_symbols=True, lam=1e-4, accumulate=True)
    _same(a3, b3, "third call")
    for k in ("fit", "rate", "hist", "symbols"):          # (the gradient buffers start from fresh random values)
        _same({k: a[k]}, {k: b3[k]}, "third call against the first")


def test_noalloc_rejects_what_does_not_fit_and_bad_arguments():
    L = gg.lib()
    P = 0x10000
    cap = 16 << 20
    # a bucket whose workspace would exceed the array: refused before any launch (fake pointers are never touched)
    big = np.array([0, 1 << 36], dtype=np.int64)
    assert gg.workspace_bytes(1 << 36, 1) > cap
    assert L.gg_fused_segmented_noalloc(P, 0, big.ctypes.data, 1, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, None) == -4
    # the documented capacity holds
    assert gg.workspace_bytes(1 << 31, 4096) <= cap
    ok = np.array([0, 10, 20], dtype=np.int64)
    assert L.gg_fused_segmented_noalloc(P, 7, ok.ctypes.data, 2, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, None) == -2
    assert L.gg_fused_segmented_noalloc(None, 0, ok.ctypes.data, 2, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, None) == -1
    assert L.gg_fused_segmented_noalloc(P, 0, ok.ctypes.data, 2, 16.0, None, 99, 0, 0, None, None, 0.0, None, 0, P, P, None) == -1
    bad = np.array([0, 10, 5], dtype=np.int64)
    assert L.gg_fused_segmented_noalloc(P, 0, bad.ctypes.data, 2, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, None) == -3
