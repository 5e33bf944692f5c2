"""ctypes binding of libgg.so: same names as the C ABI (include/gg.h), argument marshalling only.

Tensors are torch tensors on the GPU (float32 or bfloat16 inputs).  Result records come back as
device byte tensors; `fit_records` / `rate_records` copy them to the host as numpy structured
arrays.  All work is enqueued on torch's current stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

GG_F32, GG_BF16 = 0, 1
GG_FLOOR, GG_NEAREST_EVEN = 0, 1
GG_EG_TILE = 256            # symbols per entry of the decoding index (GG_EG_TILE in gg.h)
GG_F_EMPTY, GG_F_DEGENERATE, GG_F_BETA_CLAMPED_LO, GG_F_BETA_CLAMPED_HI, GG_F_NONFINITE, GG_F_SATURATED = \
    1, 2, 4, 8, 16, 32

# host views of gg_fit_t (40 bytes) and gg_rate_t (48 bytes)
FIT_DTYPE = np.dtype([("sum_abs", "<f8"), ("sum_sq", "<f8"), ("n", "<u8"), ("beta", "<f4"), ("alpha", "<f4"),
                      ("flags", "<u4"), ("_pad", "<u4")])
RATE_DTYPE = np.dtype([("eg_bits", "<u8"), ("n", "<u8"), ("n_clamped", "<u8"), ("entropy_bits", "<f8"),
                       ("u_max", "<u4"), ("fl_bits", "<u4"), ("delta", "<f4"), ("flags", "<u4")])
assert FIT_DTYPE.itemsize == 40 and RATE_DTYPE.itemsize == 48

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class GGError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().gg_strerror(code).decode()} ({code})")


def lib_path() -> str:
    return os.path.join(_HERE, "libgg.so")


def lib():
    """The loaded libgg.so.  Raises if it has not been built: there is no fallback path."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2506_00486_amd.build` "
                               "(or __graft_entry__.build()); libgg has no CPU fallback")
        L = C.CDLL(path)
        vp, i32, i64, u32, u64, f32, f64, sz = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_float,
                                                C.c_double, C.c_size_t)
        ci = C.c_int
        sig = {
            "gg_strerror": (C.c_char_p, [ci]),
            "gg_workspace_bytes": (ci, [i64, i32, i32, C.POINTER(sz)]),
            "gg_fit": (ci, [vp, ci, i64, vp, vp, sz, vp]),
            "gg_fit_segmented": (ci, [vp, ci, vp, i32, vp, vp, sz, vp]),
            "gg_fit_rows": (ci, [vp, ci, i64, i64, vp, vp, vp, sz, vp]),
            "gg_quantize_rate": (ci, [vp, ci, i64, f32, ci, ci, i32, vp, vp, vp, vp, sz, vp]),
            "gg_quantize_rate_segmented": (ci, [vp, ci, vp, i32, vp, ci, ci, i32, vp, vp, vp, vp, sz, vp]),
            "gg_quantize_rate_rows": (ci, [vp, ci, i64, i64, vp, ci, ci, vp, vp, vp, sz, vp]),
            "gg_delta_from_fit": (ci, [vp, i32, f32, vp, vp]),
            "gg_penalty_grad": (ci, [vp, ci, i64, f32, f32, f32, vp, ci, vp]),
            "gg_penalty_grad_segmented": (ci, [vp, ci, vp, i32, vp, f32, vp, ci, vp, sz, vp]),
            "gg_sample": (ci, [vp, ci, i64, f32, f32, u64, u32, u64, vp]),
            "gg_philox_words": (ci, [vp, i64, u64, u32, u64, u32, vp]),
            "gg_init_alpha": (f64, [i64, f64, f64]),
            "gg_compression_ratio": (f64, [f64, f64]),
            "gg_fused_segmented": (ci, [vp, ci, vp, i32, f32, vp, ci, ci, i32, vp, vp, f32, vp, ci, vp, vp, vp, sz, vp]),
            "gg_fused_segmented_noalloc": (ci, [vp, ci, vp, i32, f32, vp, ci, ci, i32, vp, vp, f32, vp, ci, vp, vp, vp]),
            "gg_fused_rows": (ci, [vp, ci, i64, i64, f32, vp, ci, ci, vp, f32, vp, ci, vp, vp, vp, vp, sz, vp]),
            "gg_rate_grad": (ci, [vp, ci, i64, f32, ci, i64, f32, vp, ci, vp]),
            "gg_gct_update": (ci, [vp, vp, vp, i64, f32, f32, f32, f32, ci, i64, ci, vp]),
            "gg_gct_update_segmented": (ci, [vp, vp, vp, vp, i32, vp, f32, f32, f32, ci, ci, vp, sz, vp]),
            "gg_eg_workspace_bytes": (ci, [i64, C.POINTER(sz)]),
            "gg_eg_encode": (ci, [vp, i64, ci, vp, u64, vp, vp, vp]),
            "gg_eg_encode_tensor": (ci, [vp, ci, i64, f32, ci, ci, vp, u64, vp, vp, vp]),
            "gg_eg_encode_segmented": (ci, [vp, ci, vp, i32, vp, ci, ci, vp, u64, vp, vp, vp, sz, vp]),
            "gg_eg_decode": (ci, [vp, vp, i64, ci, vp, vp]),
            "gg_eg_decode_dequant": (ci, [vp, vp, i64, ci, f32, vp, ci, vp]),
            "gg_eg_decode_dequant_segmented": (ci, [vp, vp, vp, i32, ci, vp, vp, ci, vp, sz, vp]),
            "gg_huffman_mean_bits": (ci, [vp, i32, C.POINTER(f64)]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _LIB = L
    return _LIB


# ---- marshalling helpers ------------------------------------------------------------------------
def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GG_F32
    if t.dtype == torch.bfloat16:
        return GG_BF16
    raise TypeError(f"libgg takes float32 or bfloat16 tensors, got {t.dtype}")


def _dev(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libgg needs contiguous tensors in GPU memory")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _f32(v) -> float:
    return float(np.float32(v))


def _check(code: int, where: str):
    if code != 0:
        raise GGError(code, where)


def _offsets(offsets: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))


def workspace_bytes(n_total: int, n_units: int = 1, nbins: int = 0) -> int:
    out = C.c_size_t(0)
    _check(lib().gg_workspace_bytes(int(n_total), int(n_units), int(nbins), C.byref(out)), "gg_workspace_bytes")
    return out.value


class Workspace:
    """A caller-owned device scratch buffer sized by gg_workspace_bytes."""

    def __init__(self, n_total: int, n_units: int = 1, nbins: int = 0, device="cuda"):
        self.bytes = workspace_bytes(n_total, n_units, nbins)
        self.buf = torch.empty(self.bytes, dtype=torch.uint8, device=device)

    @property
    def ptr(self) -> int:
        return self.buf.data_ptr()


def _records(n: int, itemsize: int, device) -> torch.Tensor:
    return torch.empty(max(n, 1) * itemsize, dtype=torch.uint8, device=device)


def fit_records(t: torch.Tensor, n: Optional[int] = None) -> np.ndarray:
    a = t.cpu().numpy().view(FIT_DTYPE)
    return a if n is None else a[:n]


def rate_records(t: torch.Tensor, n: Optional[int] = None) -> np.ndarray:
    a = t.cpu().numpy().view(RATE_DTYPE)
    return a if n is None else a[:n]


# ---- entry points (names and argument order follow include/gg.h) --------------------------------
def gg_fit(x: torch.Tensor, ws: Workspace, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    out = out if out is not None else _records(1, 40, x.device)
    _check(lib().gg_fit(_dev(x), _dtype_code(x), x.numel(), _dev(out), ws.ptr, ws.bytes, _stream()), "gg_fit")
    return out


def gg_fit_segmented(x: torch.Tensor, offsets, ws: Workspace, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    off = _offsets(offsets)
    S = off.size - 1
    out = out if out is not None else _records(S, 40, x.device)
    _check(lib().gg_fit_segmented(_dev(x), _dtype_code(x), off.ctypes.data, S, _dev(out), ws.ptr, ws.bytes, _stream()),
           "gg_fit_segmented")
    return out


def gg_fit_rows(x: torch.Tensor, rows: int, cols: int, ws: Workspace, want_total: bool = False):
    out = _records(rows, 40, x.device)
    total = _records(1, 40, x.device) if want_total else None
    _check(lib().gg_fit_rows(_dev(x), _dtype_code(x), rows, cols, _dev(out), _dev(total), ws.ptr, ws.bytes, _stream()),
           "gg_fit_rows")
    return (out, total) if want_total else out


def gg_quantize_rate(x: torch.Tensor, delta: float, ws: Workspace, eg_k: int = 0, round_mode: int = GG_FLOOR,
                     nbins: int = 0, want_symbols: bool = False, out: Optional[torch.Tensor] = None,
                     hist: Optional[torch.Tensor] = None, symbols: Optional[torch.Tensor] = None):
    """Returns (rate record tensor, hist uint64-as-int64 tensor or None, symbols int32 tensor or None).
    `out`, `hist`, `symbols`: buffers of the caller to write into instead of new ones."""
    if nbins > 0 and hist is None:
        hist = torch.empty(nbins, dtype=torch.int64, device=x.device)
    sym = symbols if symbols is not None else (torch.empty(x.numel(), dtype=torch.int32, device=x.device) if want_symbols else None)
    out = out if out is not None else _records(1, 48, x.device)
    _check(lib().gg_quantize_rate(_dev(x), _dtype_code(x), x.numel(), _f32(delta), eg_k, round_mode, nbins, _dev(hist),
                                  _dev(sym), _dev(out), ws.ptr, ws.bytes, _stream()), "gg_quantize_rate")
    return out, hist, sym


def gg_quantize_rate_segmented(x: torch.Tensor, offsets, delta: torch.Tensor, ws: Workspace, eg_k: int = 0,
                               round_mode: int = GG_FLOOR, nbins: int = 0, want_symbols: bool = False):
    off = _offsets(offsets)
    S = off.size - 1
    hist = torch.empty(max(S, 1) * nbins, dtype=torch.int64, device=x.device) if nbins > 0 else None
    sym = torch.empty(x.numel(), dtype=torch.int32, device=x.device) if want_symbols else None
    out = _records(S, 48, x.device)
    _check(lib().gg_quantize_rate_segmented(_dev(x), _dtype_code(x), off.ctypes.data, S, _dev(delta), eg_k, round_mode,
                                            nbins, _dev(hist), _dev(sym), _dev(out), ws.ptr, ws.bytes, _stream()),
           "gg_quantize_rate_segmented")
    return out, hist, sym


def gg_quantize_rate_rows(x: torch.Tensor, rows: int, cols: int, delta: torch.Tensor, ws: Workspace, eg_k: int = 0,
                          round_mode: int = GG_FLOOR, want_symbols: bool = False):
    sym = torch.empty(x.numel(), dtype=torch.int32, device=x.device) if want_symbols else None
    out = _records(rows, 48, x.device)
    _check(lib().gg_quantize_rate_rows(_dev(x), _dtype_code(x), rows, cols, _dev(delta), eg_k, round_mode, _dev(sym),
                                       _dev(out), ws.ptr, ws.bytes, _stream()), "gg_quantize_rate_rows")
    return out, sym


def gg_delta_from_fit(fit: torch.Tensor, S: int, delta_div: float) -> torch.Tensor:
    out = torch.empty(max(S, 1), dtype=torch.float32, device=fit.device)
    _check(lib().gg_delta_from_fit(_dev(fit), S, _f32(delta_div), _dev(out), _stream()), "gg_delta_from_fit")
    return out


def gg_penalty_grad(w: torch.Tensor, alpha: float, beta: float, lam: float, grad: Optional[torch.Tensor] = None,
                    accumulate: bool = False) -> torch.Tensor:
    if grad is None:
        grad = torch.empty(w.numel(), dtype=torch.float32, device=w.device)
    _check(lib().gg_penalty_grad(_dev(w), _dtype_code(w), w.numel(), _f32(alpha), _f32(beta), _f32(lam), _dev(grad),
                                 int(bool(accumulate)), _stream()), "gg_penalty_grad")
    return grad


def gg_penalty_grad_segmented(w: torch.Tensor, offsets, fit: torch.Tensor, lam: float, ws: Workspace,
                              grad: Optional[torch.Tensor] = None, accumulate: bool = False) -> torch.Tensor:
    off = _offsets(offsets)
    S = off.size - 1
    if grad is None:
        grad = torch.empty(w.numel(), dtype=torch.float32, device=w.device)
    _check(lib().gg_penalty_grad_segmented(_dev(w), _dtype_code(w), off.ctypes.data, S, _dev(fit), _f32(lam), _dev(grad),
                                           int(bool(accumulate)), ws.ptr, ws.bytes, _stream()),
           "gg_penalty_grad_segmented")
    return grad


def gg_sample(n: int, alpha: float, beta: float, seed: int, stream_id: int = 0, offset: int = 0,
              dtype=torch.float32, device="cuda", out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(n, dtype=dtype, device=device)
    _check(lib().gg_sample(_dev(out), _dtype_code(out), n, _f32(alpha), _f32(beta), int(seed), int(stream_id),
                           int(offset), _stream()), "gg_sample")
    return out


def gg_philox_words(n: int, seed: int, stream_id: int = 0, offset: int = 0, attempt: int = 0, device="cuda"):
    out = torch.empty(4 * max(n, 1), dtype=torch.int32, device=device)
    _check(lib().gg_philox_words(_dev(out), n, int(seed), int(stream_id), int(offset), int(attempt), _stream()),
           "gg_philox_words")
    return out[: 4 * n]


def gg_init_alpha(d_in: int, shape: float, xi: float = 1.0) -> float:
    return lib().gg_init_alpha(int(d_in), float(shape), float(xi))


def gg_compression_ratio(mean_bits: float, fl_bits: float) -> float:
    return lib().gg_compression_ratio(float(mean_bits), float(fl_bits))


def gg_fused_segmented(x: torch.Tensor, offsets, ws: Workspace, delta_div: float = 16.0,
                       delta: Optional[torch.Tensor] = None, eg_k: int = 0, round_mode: int = GG_FLOOR,
                       nbins: int = 0, want_symbols: bool = False, lam: float = 0.0,
                       grad: Optional[torch.Tensor] = None, accumulate: bool = False, want_rate: bool = True,
                       fit: Optional[torch.Tensor] = None, rate: Optional[torch.Tensor] = None,
                       hist: Optional[torch.Tensor] = None):
    """Returns dict(fit=, rate=, hist=, symbols=, grad=) of device tensors (None where not requested).
    `fit`, `rate`, `hist`: buffers of the caller to write into instead of new ones."""
    off = _offsets(offsets)
    S = off.size - 1
    fit = fit if fit is not None else _records(S, 40, x.device)
    if want_rate and rate is None:
        rate = _records(S, 48, x.device)
    if not (nbins > 0 and want_rate):
        hist = None
    elif hist is None:
        hist = torch.empty(max(S, 1) * nbins, dtype=torch.int64, device=x.device)
    sym = torch.empty(x.numel(), dtype=torch.int32, device=x.device) if (want_symbols and want_rate) else None
    _check(lib().gg_fused_segmented(_dev(x), _dtype_code(x), off.ctypes.data, S, _f32(delta_div), _dev(delta), eg_k,
                                    round_mode, nbins if hist is not None else 0, _dev(hist), _dev(sym), _f32(lam),
                                    _dev(grad), int(bool(accumulate)), _dev(fit), _dev(rate) if want_rate else None,
                                    ws.ptr, ws.bytes, _stream()), "gg_fused_segmented")
    return dict(fit=fit, rate=rate if want_rate else None, hist=hist, symbols=sym, grad=grad)


def gg_fused_segmented_noalloc(x: torch.Tensor, offsets, fit: torch.Tensor, rate: Optional[torch.Tensor] = None,
                               delta_div: float = 16.0, delta: Optional[torch.Tensor] = None, eg_k: int = 0,
                               round_mode: int = GG_FLOOR, nbins: int = 0, hist: Optional[torch.Tensor] = None,
                               symbols: Optional[torch.Tensor] = None, lam: float = 0.0,
                               grad: Optional[torch.Tensor] = None, accumulate: bool = False) -> None:
    """The whole pass with the library's own scratch memory.  Every buffer, outputs included, is the caller's:
    this wrapper creates no tensor, so the call allocates nothing on either side."""
    off = _offsets(offsets)
    _check(lib().gg_fused_segmented_noalloc(_dev(x), _dtype_code(x), off.ctypes.data, off.size - 1, _f32(delta_div),
                                            _dev(delta), eg_k, round_mode, nbins, _dev(hist), _dev(symbols), _f32(lam),
                                            _dev(grad), int(bool(accumulate)), _dev(fit), _dev(rate), _stream()),
           "gg_fused_segmented_noalloc")


def gg_fused_rows(x: torch.Tensor, rows: int, cols: int, ws: Workspace, delta_div: float = 16.0,
                  delta: Optional[torch.Tensor] = None, eg_k: int = 0, round_mode: int = GG_FLOOR,
                  want_symbols: bool = False, lam: float = 0.0, grad: Optional[torch.Tensor] = None,
                  accumulate: bool = False, want_rate: bool = True, want_total: bool = False,
                  fit: Optional[torch.Tensor] = None, total: Optional[torch.Tensor] = None,
                  rate: Optional[torch.Tensor] = None):
    """`fit`, `total`, `rate`: buffers of the caller to write into instead of new ones."""
    fit = fit if fit is not None else _records(rows, 40, x.device)
    total = (total if total is not None else _records(1, 40, x.device)) if want_total else None
    rate = (rate if rate is not None else _records(rows, 48, x.device)) if want_rate else None
    sym = torch.empty(x.numel(), dtype=torch.int32, device=x.device) if (want_symbols and want_rate) else None
    _check(lib().gg_fused_rows(_dev(x), _dtype_code(x), rows, cols, _f32(delta_div), _dev(delta), eg_k, round_mode,
                               _dev(sym), _f32(lam), _dev(grad), int(bool(accumulate)), _dev(fit), _dev(total),
                               _dev(rate), ws.ptr, ws.bytes, _stream()), "gg_fused_rows")
    return dict(fit=fit, total=total, rate=rate, symbols=sym, grad=grad)


# ---- companions of the pass inside the training algorithms --------------------------------------
def gg_rate_grad(x: torch.Tensor, delta: float, eg_k: int = 0, n_rate: Optional[int] = None, scale: float = 1.0,
                 grad: Optional[torch.Tensor] = None, accumulate: bool = False) -> torch.Tensor:
    if grad is None:
        grad = torch.empty(x.numel(), dtype=torch.float32, device=x.device)
    _check(lib().gg_rate_grad(_dev(x), _dtype_code(x), x.numel(), _f32(delta), eg_k,
                              x.numel() if n_rate is None else int(n_rate), _f32(scale), _dev(grad),
                              int(bool(accumulate)), _stream()), "gg_rate_grad")
    return grad


def gg_gct_update(w: torch.Tensor, g: torch.Tensor, ghat_prev: torch.Tensor, eta: float, lam: float, eps: float,
                  delta: float, eg_k: int = 0, n_rate: Optional[int] = None, first_step: bool = False) -> None:
    for t in (w, g, ghat_prev):
        if t.dtype != torch.float32:
            raise TypeError("gg_gct_update works on float32 tensors")
    _check(lib().gg_gct_update(_dev(w), _dev(g), _dev(ghat_prev), w.numel(), _f32(eta), _f32(lam), _f32(eps),
                               _f32(delta), eg_k, w.numel() if n_rate is None else int(n_rate), int(bool(first_step)),
                               _stream()), "gg_gct_update")


def gg_gct_update_segmented(w: torch.Tensor, g: torch.Tensor, ghat_prev: torch.Tensor, offsets, delta: torch.Tensor,
                            eta: float, lam: float, eps: float, ws: Workspace, eg_k: int = 0,
                            first_step: bool = False) -> None:
    off = _offsets(offsets)
    for t in (w, g, ghat_prev):
        if t.dtype != torch.float32:
            raise TypeError("gg_gct_update_segmented works on float32 tensors")
    _check(lib().gg_gct_update_segmented(_dev(w), _dev(g), _dev(ghat_prev), off.ctypes.data, off.size - 1, _dev(delta),
                                         _f32(eta), _f32(lam), _f32(eps), eg_k, int(bool(first_step)), ws.ptr, ws.bytes,
                                         _stream()), "gg_gct_update_segmented")


def gg_eg_encode(symbols: torch.Tensor, eg_k: int = 0, capacity_bytes: Optional[int] = None, buffers=None):
    """Returns (stream uint8 tensor, index int64 tensor of bit offsets, total_bits int).  Without a capacity the
    stream is sized for the worst case of 8 bytes per symbol.  `buffers` = (stream, workspace, total) from an
    earlier call's `eg_buffers` reuses device memory and skips the read-back of the total (returned as None)."""
    n = symbols.numel()
    if buffers is None:
        stream, work, total = eg_buffers(n, capacity_bytes, symbols.device)
    else:
        stream, work, total = buffers
    _check(lib().gg_eg_encode(_dev(symbols), n, eg_k, _dev(stream), stream.numel(), _dev(work), _dev(total), _stream()),
           "gg_eg_encode")
    tiles = (n + GG_EG_TILE - 1) // GG_EG_TILE
    return stream, work[: tiles + 1], (int(total.item()) if buffers is None else None)


def gg_eg_encode_tensor(x: torch.Tensor, delta: float, eg_k: int = 0, round_mode: int = GG_FLOOR,
                        capacity_bytes: Optional[int] = None, buffers=None):
    """Quantise and encode in one go (no symbol array): returns (stream, index, total_bits) as gg_eg_encode."""
    n = x.numel()
    if buffers is None:
        stream, work, total = eg_buffers(n, capacity_bytes, x.device)
    else:
        stream, work, total = buffers
    _check(lib().gg_eg_encode_tensor(_dev(x), _dtype_code(x), n, _f32(delta), round_mode, eg_k, _dev(stream),
                                     stream.numel(), _dev(work), _dev(total), _stream()), "gg_eg_encode_tensor")
    tiles = (n + GG_EG_TILE - 1) // GG_EG_TILE
    return stream, work[: tiles + 1], (int(total.item()) if buffers is None else None)


def gg_eg_encode_segmented(x: torch.Tensor, offsets: Sequence[int], delta: torch.Tensor, ws: Workspace, eg_k: int = 0,
                           round_mode: int = GG_FLOOR, capacity_bytes: Optional[int] = None, buffers=None):
    """One stream for a flat bucket with a step per unit (device tensor `delta`); returns as gg_eg_encode."""
    off = _offsets(offsets)
    n = int(off[-1]) if off.size else 0
    if buffers is None:
        stream, work, total = eg_buffers(n, capacity_bytes, x.device)
    else:
        stream, work, total = buffers
    _check(lib().gg_eg_encode_segmented(_dev(x), _dtype_code(x), off.ctypes.data, off.size - 1, _dev(delta), round_mode, eg_k,
                                        _dev(stream), stream.numel(), _dev(work), _dev(total), ws.ptr, ws.bytes, _stream()),
           "gg_eg_encode_segmented")
    tiles = (n + GG_EG_TILE - 1) // GG_EG_TILE
    return stream, work[: tiles + 1], (int(total.item()) if buffers is None else None)


def eg_buffers(n: int, capacity_bytes: Optional[int] = None, device="cuda"):
    """Device buffers for gg_eg_encode: (stream, index workspace, total)."""
    out = C.c_size_t(0)
    _check(lib().gg_eg_workspace_bytes(n, C.byref(out)), "gg_eg_workspace_bytes")
    work = torch.empty(out.value // 8, dtype=torch.int64, device=device)
    cap = (8 * n + 4) if capacity_bytes is None else int(capacity_bytes)
    cap = (cap + 3) // 4 * 4
    stream = torch.empty(cap, dtype=torch.uint8, device=device)
    total = torch.zeros(1, dtype=torch.int64, device=device)
    return stream, work, total


def gg_eg_decode(stream: torch.Tensor, index: torch.Tensor, n: int, eg_k: int = 0, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty(n, dtype=torch.int32, device=stream.device)
    _check(lib().gg_eg_decode(_dev(stream), _dev(index), n, eg_k, _dev(out), _stream()), "gg_eg_decode")
    return out


def gg_eg_decode_dequant(stream: torch.Tensor, index: torch.Tensor, n: int, delta: float, eg_k: int = 0,
                         out: Optional[torch.Tensor] = None, accumulate: bool = False) -> torch.Tensor:
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs the tensor to add to")
        out = torch.empty(n, dtype=torch.float32, device=stream.device)
    _check(lib().gg_eg_decode_dequant(_dev(stream), _dev(index), n, eg_k, _f32(delta), _dev(out), int(bool(accumulate)),
                                      _stream()), "gg_eg_decode_dequant")
    return out


def gg_eg_decode_dequant_segmented(stream: torch.Tensor, index: torch.Tensor, offsets, delta: torch.Tensor, ws: Workspace,
                                   eg_k: int = 0, out: Optional[torch.Tensor] = None, accumulate: bool = False) -> torch.Tensor:
    off = _offsets(offsets)
    n = int(off[-1])
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs the tensor to add to")
        out = torch.empty(n, dtype=torch.float32, device=stream.device)
    _check(lib().gg_eg_decode_dequant_segmented(_dev(stream), _dev(index), off.ctypes.data, off.size - 1, eg_k, _dev(delta),
                                                _dev(out), int(bool(accumulate)), ws.ptr, ws.bytes, _stream()),
           "gg_eg_decode_dequant_segmented")
    return out


def gg_huffman_mean_bits(hist) -> float:
    h = np.ascontiguousarray(np.asarray(hist.cpu() if isinstance(hist, torch.Tensor) else hist)).view(np.uint64)
    out = C.c_double(0.0)
    _check(lib().gg_huffman_mean_bits(h.ctypes.data, h.size, C.byref(out)), "gg_huffman_mean_bits")
    return out.value
