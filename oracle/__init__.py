"""ctypes front-end of the C oracle (oracle/gg_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never imports the product package and shares nothing with it.
Arrays are numpy: float32 for fp32 data, uint16 holding raw bits for bf16 data.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
ROUND_FLOOR, ROUND_NEAREST_EVEN = 0, 1
EMPTY, DEGENERATE, BETA_CLAMPED_LO, BETA_CLAMPED_HI, NONFINITE, SATURATED = 1, 2, 4, 8, 16, 32
BETA_MIN, BETA_MAX = 0.05, 20.0


class Fit(C.Structure):
    _fields_ = [("sum_abs", C.c_double), ("sum_sq", C.c_double), ("n", C.c_uint64),
                ("beta", C.c_double), ("alpha", C.c_double), ("flags", C.c_uint32)]

    def __repr__(self):
        return (f"Fit(n={self.n}, sum_abs={self.sum_abs!r}, sum_sq={self.sum_sq!r}, "
                f"beta={self.beta!r}, alpha={self.alpha!r}, flags={self.flags})")


class Rate(C.Structure):
    _fields_ = [("eg_bits", C.c_uint64), ("n", C.c_uint64), ("n_clamped", C.c_uint64),
                ("entropy_bits", C.c_double), ("u_max", C.c_uint32), ("fl_bits", C.c_uint32),
                ("flags", C.c_uint32)]

    def __repr__(self):
        return (f"Rate(n={self.n}, eg_bits={self.eg_bits}, u_max={self.u_max}, fl_bits={self.fl_bits}, "
                f"n_clamped={self.n_clamped}, entropy_bits={self.entropy_bits!r}, flags={self.flags})")


_lib = None


def load(path: str):
    """Opens a build of gg_oracle.c and declares its signatures (the tests also load altered builds this way)."""
    L = C.CDLL(path)
    vp, i32, i64, u32, u64, f32, f64 = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64,
                                        C.c_float, C.c_double)
    L.orc_rho.restype = f64
    L.orc_rho.argtypes = [f64]
    L.orc_solve_beta.restype = f64
    L.orc_solve_beta.argtypes = [f64, C.POINTER(u32)]
    L.orc_alpha_from_m2.restype = f64
    L.orc_alpha_from_m2.argtypes = [f64, f64]
    L.orc_init_alpha.restype = f64
    L.orc_init_alpha.argtypes = [i64, f64, f64]
    L.orc_moments.restype = None
    L.orc_moments.argtypes = [vp, C.c_int, i64, C.POINTER(f64), C.POINTER(f64)]
    L.orc_fit_from_moments.restype = None
    L.orc_fit_from_moments.argtypes = [f64, f64, u64, C.POINTER(Fit)]
    L.orc_fit.restype = None
    L.orc_fit.argtypes = [vp, C.c_int, i64, C.POINTER(Fit)]
    L.orc_quantize_one.restype = i32
    L.orc_quantize_one.argtypes = [f32, f32, C.c_int, C.POINTER(u32)]
    L.orc_map.restype = u32
    L.orc_map.argtypes = [i32]
    L.orc_eg_len.restype = u32
    L.orc_eg_len.argtypes = [u32, C.c_int]
    L.orc_quantize_rate.restype = None
    L.orc_quantize_rate.argtypes = [vp, C.c_int, i64, f32, C.c_int, C.c_int, i32, vp, vp, C.POINTER(Rate)]
    L.orc_penalty_grad.restype = None
    L.orc_penalty_grad.argtypes = [vp, C.c_int, i64, f32, f32, f32, vp, C.c_int]
    L.orc_philox4x32_10.restype = None
    L.orc_philox4x32_10.argtypes = [C.POINTER(u32), C.POINTER(u32), C.POINTER(u32)]
    L.orc_sample.restype = None
    L.orc_sample.argtypes = [vp, C.c_int, i64, f32, f32, u64, u32, u64]
    L.orc_round_bf16.restype = None
    L.orc_round_bf16.argtypes = [vp, i64, vp]
    L.orc_sample_attempts.restype = u64
    L.orc_sample_attempts.argtypes = [i64, f32, u64, u32, u64]
    L.orc_fused_segmented.restype = None
    L.orc_fused_segmented.argtypes = [vp, C.c_int, vp, i32, f32, vp, C.c_int, C.c_int, f32, vp, C.c_int,
                                      C.POINTER(Fit), C.POINTER(Rate)]
    L.orc_gct_update.restype = None
    L.orc_gct_update.argtypes = [vp, vp, vp, i64, f32, f32, f32, f32, C.c_int, i64, C.c_int]
    L.orc_eg_encode.restype = u64
    L.orc_eg_encode.argtypes = [vp, i64, C.c_int, vp, u64]
    L.orc_eg_decode.restype = i64
    L.orc_eg_decode.argtypes = [vp, u64, C.c_int, vp, i64]
    L.orc_dequantize.restype = None
    L.orc_dequantize.argtypes = [vp, i64, f32, vp, C.c_int]
    L.orc_huffman_mean_bits.restype = f64
    L.orc_huffman_mean_bits.argtypes = [vp, i32]
    L.orc_rate_grad.restype = None
    L.orc_rate_grad.argtypes = [vp, C.c_int, i64, f32, C.c_int, i64, f32, vp, C.c_int]
    L.orc_compression_ratio.restype = f64
    L.orc_compression_ratio.argtypes = [f64, f64]
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load(_build.build(force=False))
    return _lib


def _f32(v) -> float:
    """Round to fp32, return as a Python float (what ctypes' c_float accepts)."""
    return float(np.asarray(v, dtype=np.float32))


def _dtype_of(x: np.ndarray) -> int:
    if x.dtype == np.float32:
        return F32
    if x.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle input must be float32 or uint16 (bf16 bits), got {x.dtype}")


def _flat(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x).reshape(-1)
    return x


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def rho(beta: float) -> float:
    return lib().orc_rho(float(beta))


def solve_beta(r: float):
    fl = C.c_uint32(0)
    b = lib().orc_solve_beta(float(r), C.byref(fl))
    return b, fl.value


def alpha_from_m2(m2: float, beta: float) -> float:
    return lib().orc_alpha_from_m2(float(m2), float(beta))


def init_alpha(d_in: int, shape: float, xi: float = 1.0) -> float:
    return lib().orc_init_alpha(int(d_in), float(shape), float(xi))


def moments(x: np.ndarray):
    x = _flat(x)
    s1, s2 = C.c_double(0), C.c_double(0)
    lib().orc_moments(_ptr(x), _dtype_of(x), x.size, C.byref(s1), C.byref(s2))
    return s1.value, s2.value


def fit_from_moments(sum_abs: float, sum_sq: float, n: int) -> Fit:
    out = Fit()
    lib().orc_fit_from_moments(float(sum_abs), float(sum_sq), int(n), C.byref(out))
    return out


def fit(x: np.ndarray) -> Fit:
    x = _flat(x)
    out = Fit()
    lib().orc_fit(_ptr(x), _dtype_of(x), x.size, C.byref(out))
    return out


def quantize_one(x: float, inv_delta: float, round_mode: int = ROUND_FLOOR) -> int:
    fl = C.c_uint32(0)
    return lib().orc_quantize_one(float(x), float(inv_delta), round_mode, C.byref(fl))


def map_symbol(q: int) -> int:
    return lib().orc_map(int(q))


def eg_len(u: int, k: int = 0) -> int:
    return lib().orc_eg_len(int(u), int(k))


def quantize_rate(x: np.ndarray, delta: float, eg_k: int = 0, round_mode: int = ROUND_FLOOR,
                  nbins: int = 0, want_symbols: bool = False):
    """Returns (Rate, hist or None, symbols or None)."""
    x = _flat(x)
    hist = np.zeros(nbins, dtype=np.uint64) if nbins > 0 else None
    sym = np.empty(x.size, dtype=np.int32) if want_symbols else None
    out = Rate()
    lib().orc_quantize_rate(_ptr(x), _dtype_of(x), x.size, _f32(delta), eg_k, round_mode, nbins,
                            _ptr(hist), _ptr(sym), C.byref(out))
    return out, hist, sym


def penalty_grad(w: np.ndarray, alpha: float, beta: float, lam: float, grad: np.ndarray = None,
                 accumulate: bool = False) -> np.ndarray:
    w = _flat(w)
    if grad is None:
        grad = np.zeros(w.size, dtype=np.float32)
    assert grad.dtype == np.float32 and grad.size == w.size and grad.flags.c_contiguous
    lib().orc_penalty_grad(_ptr(w), _dtype_of(w), w.size, _f32(alpha), _f32(beta),
                           _f32(lam), _ptr(grad), int(bool(accumulate)))
    return grad


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def sample(n: int, alpha: float, beta: float, seed: int, stream: int = 0, offset: int = 0,
           dtype: int = F32) -> np.ndarray:
    out = np.empty(n, dtype=np.float32 if dtype == F32 else np.uint16)
    lib().orc_sample(_ptr(out), dtype, n, _f32(alpha), _f32(beta), int(seed), int(stream),
                     int(offset))
    return out


def round_bf16(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns of fp32 values, as sample(dtype=BF16) rounds them."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    out = np.empty(x.size, dtype=np.uint16)
    lib().orc_round_bf16(_ptr(x), x.size, _ptr(out))
    return out


def sample_attempts(n: int, beta: float, seed: int, stream: int = 0, offset: int = 0) -> int:
    """Attempts the rejection step takes over the n draws that sample() makes with the same arguments."""
    return int(lib().orc_sample_attempts(n, _f32(beta), int(seed), int(stream), int(offset)))


def fused_segmented(x: np.ndarray, offsets, delta_div: float = 16.0, delta: np.ndarray = None,
                    eg_k: int = 0, round_mode: int = ROUND_FLOOR, lam: float = 0.0,
                    grad: np.ndarray = None, accumulate: bool = False):
    """Returns (list[Fit], list[Rate]) for the segments offsets[s]..offsets[s+1]."""
    x = _flat(x)
    off = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
    S = off.size - 1
    fits = (Fit * max(S, 1))()
    rates = (Rate * max(S, 1))()
    if delta is not None:
        delta = np.ascontiguousarray(delta, dtype=np.float32)
    lib().orc_fused_segmented(_ptr(x), _dtype_of(x), _ptr(off), S, _f32(delta_div), _ptr(delta),
                              eg_k, round_mode, _f32(lam), _ptr(grad), int(bool(accumulate)),
                              fits, rates)
    return list(fits)[:S], list(rates)[:S]


def gct_update(w: np.ndarray, g: np.ndarray, g_hat_prev: np.ndarray, eta: float, lam: float, eps: float,
               inv_delta: float, eg_k: int, n_rate: int, first_step: bool):
    """In place on w and g_hat_prev (float32, contiguous)."""
    for a in (w, g, g_hat_prev):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    lib().orc_gct_update(_ptr(w), _ptr(g), _ptr(g_hat_prev), w.size, _f32(eta), _f32(lam),
                         _f32(eps), _f32(inv_delta), eg_k, int(n_rate), int(bool(first_step)))


def eg_encode(u: np.ndarray, eg_k: int = 0):
    """Returns (bytes array, n_bits)."""
    u = np.ascontiguousarray(u, dtype=np.uint32)
    cap = int(u.size) * 8 + 8  # <= 63 bits/symbol
    buf = np.zeros(cap, dtype=np.uint8)
    nbits = lib().orc_eg_encode(_ptr(u), u.size, eg_k, _ptr(buf), cap)
    return buf[: (nbits + 7) // 8].copy(), int(nbits)


def eg_decode(buf: np.ndarray, n_bits: int, eg_k: int, max_n: int) -> np.ndarray:
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    out = np.empty(max_n, dtype=np.uint32)
    cnt = lib().orc_eg_decode(_ptr(buf), int(n_bits), eg_k, _ptr(out), max_n)
    if cnt < 0:
        raise ValueError("truncated Exp-Golomb stream")
    return out[:cnt]


def dequantize(q: np.ndarray, delta: float, out: np.ndarray = None, accumulate: bool = False) -> np.ndarray:
    """out (=|+=) q * delta in fp32."""
    q = np.ascontiguousarray(q, dtype=np.int32).reshape(-1)
    if out is None:
        out = np.zeros(q.size, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == q.size and out.flags.c_contiguous
    lib().orc_dequantize(_ptr(q), q.size, _f32(delta), _ptr(out), int(bool(accumulate)))
    return out


def huffman_mean_bits(hist: np.ndarray) -> float:
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    return lib().orc_huffman_mean_bits(_ptr(hist), hist.size)


def compression_ratio(mean_bits: float, fl_bits: float) -> float:
    return lib().orc_compression_ratio(float(mean_bits), float(fl_bits))


def rate_grad(x: np.ndarray, inv_delta: float, eg_k: int, n_rate: int, scale: float = 1.0,
              grad: np.ndarray = None, accumulate: bool = False) -> np.ndarray:
    x = _flat(x)
    if grad is None:
        grad = np.zeros(x.size, dtype=np.float32)
    lib().orc_rate_grad(_ptr(x), _dtype_of(x), x.size, _f32(inv_delta), eg_k, int(n_rate), _f32(scale), _ptr(grad),
                        int(bool(accumulate)))
    return grad
