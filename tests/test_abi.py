"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header
declares, and rejects invalid arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2506_00486_amd as gg
    if not os.path.exists(gg.lib_path()):
        from paper_2506_00486_amd import build
        build.build()
    return gg


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gg_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    gg = _lib()
    names = declared_functions()
    assert len(names) >= 17
    for n in names:
        assert hasattr(gg.lib(), n), n
    # and the binding offers the same names
    for n in names:
        if n in ("gg_strerror", "gg_workspace_bytes", "gg_eg_workspace_bytes"):
            continue
        assert hasattr(gg, n), n


def test_struct_sizes_match_header():
    gg = _lib()
    assert gg.FIT_DTYPE.itemsize == 40 and gg.RATE_DTYPE.itemsize == 48
    assert gg.FIT_DTYPE.fields["beta"][1] == 24 and gg.FIT_DTYPE.fields["flags"][1] == 32
    assert gg.RATE_DTYPE.fields["u_max"][1] == 32 and gg.RATE_DTYPE.fields["delta"][1] == 40


def test_strerror_and_workspace_size():
    gg = _lib()
    L = gg.lib()
    assert L.gg_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert L.gg_strerror(code) not in (b"ok", b"unknown error")
    small = gg.workspace_bytes(1 << 20, 1)
    big = gg.workspace_bytes(1543655424, 253)
    assert 0 < small < big < 64 << 20
    out = C.c_size_t(0)
    assert L.gg_workspace_bytes(-1, 1, 0, C.byref(out)) == -1
    assert L.gg_workspace_bytes(10, -1, 0, C.byref(out)) == -1
    assert L.gg_workspace_bytes(10, 1, 0, None) == -1


def test_invalid_arguments_are_rejected_on_the_host():
    """Every call below fails validation before any launch, so no GPU is needed.  The device
    pointers are fake but well-aligned addresses that are never dereferenced."""
    gg = _lib()
    L = gg.lib()
    P = 0x10000  # aligned fake device address
    ws_bytes = gg.workspace_bytes(1 << 20, 4)
    off = np.array([0, 10, 5, 20], dtype=np.int64)  # decreasing
    ok_off = np.array([0, 10, 15, 20], dtype=np.int64)
    assert L.gg_fit(P, 7, 100, P, P, ws_bytes, None) == -2                       # dtype
    assert L.gg_fit(P, 0, -5, P, P, ws_bytes, None) == -1                        # n < 0
    assert L.gg_fit(None, 0, 100, P, P, ws_bytes, None) == -1                    # null x
    assert L.gg_fit(P + 4, 0, 100, P, P, ws_bytes, None) == -1                   # misaligned x
    assert L.gg_fit(P, 0, 100, None, P, ws_bytes, None) == -1                    # null out
    assert L.gg_fit(P, 0, 100, P, None, ws_bytes, None) == -4                    # no workspace
    assert L.gg_fit(P, 0, 1 << 20, P, P, 64, None) == -4                         # workspace too small
    assert L.gg_fit_segmented(P, 0, off.ctypes.data, 3, P, P, ws_bytes, None) == -3
    assert L.gg_fit_segmented(P, 0, None, 3, P, P, ws_bytes, None) == -1
    neg = np.array([-1, 10], dtype=np.int64)
    assert L.gg_fit_segmented(P, 0, neg.ctypes.data, 1, P, P, ws_bytes, None) == -3
    assert L.gg_fit_segmented(P, 0, ok_off.ctypes.data, (1 << 17) + 1, P, P, ws_bytes, None) == -3   # too many units
    assert L.gg_fit_rows(P, 0, -1, 10, P, None, P, ws_bytes, None) == -1
    for delta in (0.0, -1.0, float("inf"), float("nan")):
        assert L.gg_quantize_rate(P, 0, 100, delta, 0, 0, 0, None, None, P, P, ws_bytes, None) == -1
    assert L.gg_quantize_rate(P, 0, 100, 0.1, 16, 0, 0, None, None, P, P, ws_bytes, None) == -1   # k > 15
    assert L.gg_quantize_rate(P, 0, 100, 0.1, -1, 0, 0, None, None, P, P, ws_bytes, None) == -1
    assert L.gg_quantize_rate(P, 0, 100, 0.1, 0, 2, 0, None, None, P, P, ws_bytes, None) == -1    # round mode
    assert L.gg_quantize_rate(P, 0, 100, 0.1, 0, 0, 1, P, None, P, P, ws_bytes, None) == -1       # nbins 1
    assert L.gg_quantize_rate(P, 0, 100, 0.1, 0, 0, 65537, P, None, P, P, ws_bytes, None) == -1
    assert L.gg_quantize_rate(P, 0, 100, 0.1, 0, 0, 64, None, None, P, P, ws_bytes, None) == -1   # nbins without hist
    assert L.gg_quantize_rate(P, 0, 100, 0.1, 0, 0, 0, None, P + 4, P, P, ws_bytes, None) == -1   # misaligned symbols
    assert L.gg_quantize_rate_segmented(P, 0, ok_off.ctypes.data, 3, None, 0, 0, 0, None, None, P, P, ws_bytes,
                                        None) == -1                                                # no steps
    assert L.gg_penalty_grad(P, 0, 100, 0.0, 1.0, 1e-4, P, 0, None) == -1                          # alpha 0
    assert L.gg_penalty_grad(P, 0, 100, 0.1, -1.0, 1e-4, P, 0, None) == -1
    assert L.gg_penalty_grad(P, 0, 100, 0.1, 1.0, 1e-4, None, 0, None) == -1
    assert L.gg_sample(P, 0, 100, 0.1, 0.01, 1, 0, 0, None) == -1                                  # beta below range
    assert L.gg_sample(P, 0, 100, -0.1, 1.0, 1, 0, 0, None) == -1
    assert L.gg_sample(P, 3, 100, 0.1, 1.0, 1, 0, 0, None) == -2
    assert L.gg_sample(None, 0, 100, 0.1, 1.0, 1, 0, 0, None) == -1
    assert L.gg_fused_segmented(P, 0, off.ctypes.data, 3, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, P,
                                ws_bytes, None) == -3
    assert L.gg_fused_segmented(P, 0, ok_off.ctypes.data, 3, 0.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, P,
                                ws_bytes, None) == -1                                              # no step source
    assert L.gg_fused_segmented(P, 0, ok_off.ctypes.data, 3, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, None, P, P,
                                ws_bytes, None) == -1                                              # no fit output
    # the order and the rounding mode are checked even when no rate is asked for (penalty-only / fit-only calls)
    for bad_k, bad_mode in ((-1, 0), (16, 0), (40, 0), (0, 2), (0, -1)):
        assert L.gg_fused_segmented(P, 0, ok_off.ctypes.data, 3, 16.0, None, bad_k, bad_mode, 0, None, None, 1e-4, P, 0, P,
                                    None, P, ws_bytes, None) == -1
        assert L.gg_fused_rows(P, 0, 4, 5, 16.0, None, bad_k, bad_mode, None, 1e-4, P, 0, P, None, None, P, ws_bytes,
                               None) == -1
    # the bucket coder covers elements 0 .. offsets[S): a gap in front of the first unit is refused
    gap_off = np.array([4, 10, 15, 20], dtype=np.int64)
    assert L.gg_eg_encode_segmented(P, 0, gap_off.ctypes.data, 3, P, 0, 0, P, 1024, P, None, P, ws_bytes, None) == -3
    assert L.gg_eg_decode_dequant_segmented(P, P, gap_off.ctypes.data, 3, 0, P, P, 0, P, ws_bytes, None) == -3
    assert L.gg_delta_from_fit(P, 3, 0.0, P, None) == -1
    # companions
    assert L.gg_rate_grad(P, 0, 100, 0.0, 0, 100, 1.0, P, 0, None) == -1                           # step 0
    assert L.gg_rate_grad(P, 0, 100, 0.1, 0, 0, 1.0, P, 0, None) == -1                             # n_rate 0
    assert L.gg_rate_grad(P, 5, 100, 0.1, 0, 100, 1.0, P, 0, None) == -2
    assert L.gg_gct_update(P, P, P, 100, 0.0, 1.0, 1e-8, 0.1, 0, 100, 0, None) == -1               # eta 0
    assert L.gg_gct_update(P, None, P, 100, 0.1, 1.0, 1e-8, 0.1, 0, 100, 0, None) == -1
    assert L.gg_gct_update_segmented(P, P, P, off.ctypes.data, 3, P, 0.1, 1.0, 1e-8, 0, 0, P, ws_bytes, None) == -3
    assert L.gg_eg_encode(P, 100, 16, P, 1024, P, None, None) == -1                                # k > 15
    assert L.gg_eg_encode(P, 100, 0, P, 1022, P, None, None) == -1                                 # size not a multiple of 4
    assert L.gg_eg_encode(P, 100, 0, P, 1024, None, None, None) == -4                              # no index buffer
    assert L.gg_eg_encode(P + 4, 100, 0, P, 1024, P, None, None) == -1                             # misaligned symbols
    assert L.gg_eg_encode(P, 100, 0, P + 2, 1024, P, None, None) == -1                             # misaligned stream
    assert L.gg_eg_encode_tensor(P, 4, 100, 0.1, 0, 0, P, 1024, P, None, None) == -2               # dtype
    assert L.gg_eg_encode_tensor(P, 0, 100, 0.0, 0, 0, P, 1024, P, None, None) == -1               # step 0
    assert L.gg_eg_encode_tensor(P, 0, 100, float("nan"), 0, 0, P, 1024, P, None, None) == -1
    assert L.gg_eg_encode_tensor(P, 0, 100, 0.1, 3, 0, P, 1024, P, None, None) == -1               # round mode
    assert L.gg_eg_encode_tensor(P + 8, 1, 100, 0.1, 0, 0, P, 1024, P, None, None) == -1           # misaligned x
    assert L.gg_eg_encode_tensor(P, 1, 100, 0.1, 0, 0, P, 1024, None, None, None) == -4
    assert L.gg_eg_encode_segmented(P, 0, off.ctypes.data, 3, P, 0, 0, P, 1024, P, None, P, ws_bytes, None) == -3
    assert L.gg_eg_encode_segmented(P, 0, ok_off.ctypes.data, 3, None, 0, 0, P, 1024, P, None, P, ws_bytes, None) == -1   # no steps
    assert L.gg_eg_encode_segmented(P, 0, ok_off.ctypes.data, 3, P, 0, 0, P, 1024, P, None, None, 0, None) == -4           # no workspace
    assert L.gg_eg_encode_segmented(P, 2, ok_off.ctypes.data, 3, P, 0, 0, P, 1024, P, None, P, ws_bytes, None) == -2
    assert L.gg_eg_decode(P, P, -1, 0, P, None) == -1
    assert L.gg_eg_decode(P + 1, P, 100, 0, P, None) == -1                                         # misaligned stream
    assert L.gg_eg_decode(P, P, 100, 0, P + 4, None) == -1                                         # misaligned output
    assert L.gg_eg_decode(P, P, 0, 0, None, None) == 0                                             # nothing to decode
    assert L.gg_eg_decode_dequant(P, P, 100, 0, 0.0, P, 0, None) == -1                            # step 0
    assert L.gg_eg_decode_dequant(P, P, 100, 0, float("inf"), P, 0, None) == -1
    assert L.gg_eg_decode_dequant(P, P, 100, 0, 0.1, P + 4, 0, None) == -1                        # misaligned output
    assert L.gg_eg_decode_dequant(P, P, 100, 16, 0.1, P, 0, None) == -1
    assert L.gg_eg_decode_dequant(P, None, 100, 0, 0.1, P, 0, None) == -1
    assert L.gg_eg_decode_dequant(P, P, 0, 0, 0.1, None, 0, None) == 0                             # nothing to decode
    assert L.gg_eg_decode_dequant_segmented(P, P, off.ctypes.data, 3, 0, P, P, 0, P, ws_bytes, None) == -3     # decreasing offsets
    assert L.gg_eg_decode_dequant_segmented(P, P, ok_off.ctypes.data, 3, 0, None, P, 0, P, ws_bytes, None) == -1  # no steps
    assert L.gg_eg_decode_dequant_segmented(P, P, ok_off.ctypes.data, 3, 0, P, P, 0, None, 0, None) == -4         # no workspace
    assert L.gg_eg_decode_dequant_segmented(P, P, ok_off.ctypes.data, 3, 16, P, P, 0, P, ws_bytes, None) == -1
    assert L.gg_eg_decode_dequant_segmented(P, P, ok_off.ctypes.data, 0, 0, None, None, 0, P, ws_bytes, None) == 0 # no units
    out = C.c_double(0)
    assert L.gg_huffman_mean_bits(None, 4, C.byref(out)) == -1


def test_sizes_beyond_the_limits_are_rejected_without_overflow():
    """Element counts whose product, chunk count or table size would not fit are refused by the host checks
    (none of these calls reaches a launch)."""
    gg = _lib()
    L = gg.lib()
    P = 0x10000
    ws_bytes = gg.workspace_bytes(1 << 20, 4)
    assert L.gg_fit_rows(P, 0, 1 << 24, 1 << 40, P, None, P, ws_bytes, None) == -1            # rows * cols overflows int64
    assert L.gg_fit_rows(P, 0, (1 << 24) + 1, 4, P, None, P, ws_bytes, None) == -1            # more rows than units allowed
    assert L.gg_fit_rows(P, 0, 1 << 24, 1 << 38, P, None, P, ws_bytes, None) == -1            # more chunks than an int32 counts
    far = np.array([0, 1 << 62], dtype=np.int64)
    assert L.gg_fit_segmented(P, 0, far.ctypes.data, 1, P, P, ws_bytes, None) == -3           # likewise for a bucket
    assert L.gg_fused_segmented(P, 0, far.ctypes.data, 1, 16.0, None, 0, 0, 0, None, None, 0.0, None, 0, P, P, P,
                                ws_bytes, None) == -3
    big = np.array([0, 1 << 40], dtype=np.int64)                                              # a legal size: the workspace is what is missing
    assert L.gg_fit_segmented(P, 0, big.ctypes.data, 1, P, P, ws_bytes, None) == -4
    out = C.c_size_t(0)
    assert L.gg_workspace_bytes(-1, 1, 0, C.byref(out)) == -1
    assert L.gg_workspace_bytes(1 << 20, -1, 0, C.byref(out)) == -1
    assert L.gg_workspace_bytes(1 << 20, 1, 0, None) == -1
    assert L.gg_workspace_bytes(1 << 40, 1 << 20, 0, C.byref(out)) == 0 and out.value > (1 << 40) // 16384 * 16
    assert L.gg_eg_workspace_bytes(-1, C.byref(out)) == -1
    assert L.gg_sample(P, 0, -1, 0.1, 1.0, 1, 0, 0, None) == -1
    assert L.gg_quantize_rate(P, 0, -1, 0.1, 0, 0, 0, None, None, P, P, ws_bytes, None) == -1
    assert L.gg_eg_encode(P, -1, 0, P, 1024, P, None, None) == -1


def test_host_helpers_match_paper_special_cases():
    gg = _lib()
    # Eq. 5 at shape 2 is He initialisation: alpha = sqrt(2 xi / d_in)
    assert gg.gg_init_alpha(4096, 2.0, 2.0) == pytest.approx((2 * 2.0 / 4096) ** 0.5, rel=1e-13)
    assert np.isnan(gg.gg_init_alpha(0, 2.0, 1.0))
    # a row of the paper's result table: EG 1.59 bits at FL 12 -> 86.75 %
    assert 100 * gg.gg_compression_ratio(1.59, 12.0) == pytest.approx(86.75, abs=0.005)


def test_huffman_mean_bits_host_helper():
    gg = _lib()
    assert gg.gg_huffman_mean_bits(np.array([1, 1, 2, 4], dtype=np.uint64)) == pytest.approx(14 / 8)   # lengths 3,3,2,1
    assert gg.gg_huffman_mean_bits(np.array([5, 5, 5, 5], dtype=np.uint64)) == 2.0
    assert gg.gg_huffman_mean_bits(np.array([0, 9, 0], dtype=np.uint64)) == 1.0
    assert gg.gg_huffman_mean_bits(np.zeros(8, dtype=np.uint64)) == 0.0
    import oracle
    rng = np.random.default_rng(0)
    h = rng.integers(0, 1000, size=5000).astype(np.uint64)
    assert gg.gg_huffman_mean_bits(h) == pytest.approx(oracle.huffman_mean_bits(h), rel=1e-12)
    out = C.c_size_t(0)
    assert gg.lib().gg_eg_workspace_bytes(4097, C.byref(out)) == 0 and out.value == (17 + 2 * 3 + 2 + 1) * 8   # 17 index tiles + 1, 3 packing tiles: offsets + 1 and sizes, one scan group


def test_empty_calls_are_ok_without_gpu_work():
    """n == 0 / S == 0 paths that return before touching the device."""
    gg = _lib()
    L = gg.lib()
    assert L.gg_sample(None, 0, 0, 0.1, 1.0, 1, 0, 0, None) == 0
    assert L.gg_philox_words(None, 0, 1, 0, 0, 0, None) == 0
    assert L.gg_delta_from_fit(None, 0, 16.0, None, None) == 0


def test_solver_curve_written_at_build_time_matches_scipy():
    """The moment-ratio curve compiled into the library (csrc/gg_solve_curve.inc, written by gen_solve_curve.py):
    every point against scipy's log-gamma (an implementation of its own), the grid against the header's range."""
    from scipy.special import gammaln
    _lib()                                                   # builds, and with it writes the curve, if absent
    path = os.path.join(ROOT, "paper_2506_00486_amd", "csrc", "gg_solve_curve.inc")
    rows = [line.strip(" {},\n").split(",") for line in open(path) if line.startswith("{")]
    curve = np.array(rows, dtype=np.float64)
    header = open(os.path.join(ROOT, "include", "gg.h")).read()
    b_min = float(re.search(r"#define GG_BETA_MIN ([0-9.]+)", header).group(1))
    b_max = float(re.search(r"#define GG_BETA_MAX ([0-9.]+)", header).group(1))
    assert curve.shape == (4097, 2)
    b = np.exp(np.linspace(np.log(b_min), np.log(b_max), 4097))
    r = 1.0 / b
    assert np.allclose(curve[:, 0], 2 * gammaln(2 * r) - gammaln(r) - gammaln(3 * r), rtol=1e-12, atol=1e-12)
    assert np.allclose(curve[:, 1], gammaln(r) - gammaln(3 * r), rtol=1e-12, atol=1e-12)
    assert np.all(np.diff(curve[:, 0]) > 0)                  # rho grows with the shape: the search relies on it
    # closed forms on the grid's neighbours of beta = 1 and 2: rho = 1/2 and 2/pi
    for beta, rho in ((1.0, 0.5), (2.0, 2.0 / np.pi)):
        assert np.interp(np.log(beta), np.log(b), curve[:, 0]) == pytest.approx(np.log(rho), abs=1e-6)
