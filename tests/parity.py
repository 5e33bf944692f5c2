"""Helpers of the GPU parity tests: compare libgg results with the oracle's, to the stated bars.

Bars (from the benchmark spec): symbols, histogram counts, bit counts, u_max, fl_bits, n, flags:
bit-exact.  Moments 1e-5 relative; beta, alpha 1e-4 relative; penalty 1e-5 relative + 1e-7
absolute; entropy 1e-9 relative (both sides evaluate it in fp64 from identical integer counts).
"""
import concurrent.futures
import os

import numpy as np

import gg_inputs
import oracle

MOMENT_RTOL = 1e-5
PARAM_RTOL = 1e-4
PEN_RTOL, PEN_ATOL = 1e-5, 1e-7
ENTROPY_RTOL = 1e-9


def host_bits(t):
    """torch tensor -> numpy array the oracle takes (float32, or uint16 bit patterns for bf16)."""
    return gg_inputs.torch_to_numpy_bits(t)


def rel_close(a, b, rtol):
    a, b = float(a), float(b)
    if a == b:
        return True
    return abs(a - b) <= rtol * max(abs(a), abs(b))


def check_fit(gpu_rec, orc: "oracle.Fit", where=""):
    assert int(gpu_rec["n"]) == orc.n, (where, "n", gpu_rec, orc)
    assert int(gpu_rec["flags"]) == orc.flags, (where, "flags", gpu_rec, orc)
    if orc.flags & oracle.NONFINITE:
        assert float(gpu_rec["beta"]) == 2.0 and float(gpu_rec["alpha"]) == 0.0
        return
    assert rel_close(gpu_rec["sum_abs"], orc.sum_abs, MOMENT_RTOL), (where, "sum_abs", gpu_rec, orc)
    assert rel_close(gpu_rec["sum_sq"], orc.sum_sq, MOMENT_RTOL), (where, "sum_sq", gpu_rec, orc)
    assert rel_close(gpu_rec["beta"], orc.beta, PARAM_RTOL), (where, "beta", gpu_rec, orc)
    assert rel_close(gpu_rec["alpha"], orc.alpha, PARAM_RTOL), (where, "alpha", gpu_rec, orc)


def check_rate(gpu_rec, orc: "oracle.Rate", where="", entropy=True):
    for k in ("eg_bits", "n", "n_clamped", "u_max", "fl_bits", "flags"):
        assert int(gpu_rec[k]) == int(getattr(orc, k)), (where, k, gpu_rec, orc)
    if entropy:
        assert rel_close(gpu_rec["entropy_bits"], orc.entropy_bits, ENTROPY_RTOL), (where, "entropy", gpu_rec, orc)


def check_penalty(gpu_grad: np.ndarray, orc_grad: np.ndarray, where="", penalty: np.ndarray = None):
    """Write mode: |gpu - oracle| <= 1e-7 + 1e-5 |oracle|.  Accumulate mode (pass the oracle's bare
    penalty as `penalty`): the sum is one fp32 add of the penalty, so the bar applies to the
    penalty's own magnitude (the sum may cancel) plus one rounding of the sum."""
    g = gpu_grad.astype(np.float64)
    o = orc_grad.astype(np.float64)
    both_inf = np.isinf(g) & np.isinf(o) & (np.sign(g) == np.sign(o))
    scale = np.abs(o)
    if penalty is not None:
        scale = np.maximum(scale, np.abs(penalty.astype(np.float64)))
    bad = ~both_inf & ~(np.abs(g - o) <= PEN_ATOL + PEN_RTOL * scale)
    assert not bad.any(), (where, int(bad.sum()), g[bad][:5], o[bad][:5])


def oracle_threads(fn, items, workers=None):
    """fn(item) for every item on a pool of host threads, results in order.  The oracle's routines are plain C
    without global state, called through ctypes (which releases the interpreter lock for the duration of the
    call), so whole segments of a large bucket are swept side by side on the host's cores -- none of the
    threads touches the GPU."""
    workers = workers or min(16, os.cpu_count() or 1)
    with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
        return list(pool.map(fn, items))
