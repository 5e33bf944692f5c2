"""Seeded synthetic inputs shared by the tests and the benchmark.

This module belongs to neither the HIP library nor the oracle and imports
neither.  It only produces input buffers: generalized-Gaussian (GG) distributed
tensors with the shapes of LLM weights, activations and flat gradient buckets,
standing in for the model tensors the paper measures (which need its datasets
and checkpoints).  Random numbers come from numpy's / torch's own generators
(torch's device generator is a Philox stream), so nothing here is code of the
method under test.

A GG variate with scale alpha and shape beta is sign * alpha * G**(1/beta) with
G ~ Gamma(1/beta, 1) drawn by the library's gamma sampler.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

try:  # torch is only needed for device-side generation
    import torch
except Exception:  # pragma: no cover
    torch = None


# ----------------------------------------------------------------------------
# numpy (host) generator: small inputs of the CPU-only tests
# ----------------------------------------------------------------------------
def gg_numpy(n: int, alpha: float, beta: float, seed: int, dtype=np.float32) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed))
    g = rng.gamma(1.0 / beta, 1.0, size=n)
    s = rng.integers(0, 2, size=n) * 2.0 - 1.0
    return (s * alpha * g ** (1.0 / beta)).astype(dtype)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (b >> 16) & 1
    r = ((b + 0x7FFF + lsb) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = 0x7FC0
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# torch generator: runs on the device the tensor will live on
# ----------------------------------------------------------------------------
def gg_torch(n: int, alpha: float, beta: float, gen: "torch.Generator", device, dtype=None,
             block: int = 1 << 27) -> "torch.Tensor":
    """n i.i.d. GG(alpha, beta) values on `device`, drawn from `gen` in blocks."""
    dtype = dtype or torch.float32
    out = torch.empty(n, dtype=dtype, device=device)
    for lo in range(0, n, block):
        m = min(block, n - lo)
        conc = torch.full((m,), 1.0 / beta, dtype=torch.float32, device=device)
        g = torch._standard_gamma(conc, generator=gen)
        del conc
        g.pow_(1.0 / beta).mul_(alpha)
        sign = torch.randint(0, 2, (m,), generator=gen, device=device, dtype=torch.int8)
        g.mul_(sign.to(torch.float32).mul_(2.0).sub_(1.0))
        out[lo:lo + m] = g.to(dtype)
        del g, sign
    return out


def torch_to_numpy_bits(t: "torch.Tensor") -> np.ndarray:
    """Host copy as float32, or as uint16 bit patterns for bf16 tensors."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


# ----------------------------------------------------------------------------
# flat-bucket layouts (element counts per tensor, in bucket order)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Segment:
    name: str
    numel: int


def transformer_layout(layers: int, hidden: int, ffn: int, vocab: int, kv_width: int | None = None,
                       lm_head: bool = False) -> List[Segment]:
    """q,k,v,o,gate,up,down,2 norms per layer, then the embedding (and an untied head)."""
    kv = hidden if kv_width is None else kv_width
    segs: List[Segment] = []
    for l in range(layers):
        segs += [Segment(f"l{l}.q", hidden * hidden), Segment(f"l{l}.k", hidden * kv),
                 Segment(f"l{l}.v", hidden * kv), Segment(f"l{l}.o", hidden * hidden),
                 Segment(f"l{l}.gate", hidden * ffn), Segment(f"l{l}.up", hidden * ffn),
                 Segment(f"l{l}.down", ffn * hidden), Segment(f"l{l}.norm1", hidden),
                 Segment(f"l{l}.norm2", hidden)]
    segs.append(Segment("embed", vocab * hidden))
    if lm_head:
        segs.append(Segment("lm_head", vocab * hidden))
    return segs


def gradient_bucket_1p5b() -> List[Segment]:
    """28 layers, hidden 1536, FFN 8960, vocab 151936, grouped-query K/V of width 256:
    253 segments, 1,543,655,424 elements."""
    return transformer_layout(28, 1536, 8960, 151936, kv_width=256)


def weights_7b() -> List[Segment]:
    """32 layers, hidden 4096, FFN 11008, vocab 32000, untied head: 290 segments."""
    return transformer_layout(32, 4096, 11008, 32000, lm_head=True)


def offsets_of(segs: Sequence[Segment]) -> np.ndarray:
    off = np.zeros(len(segs) + 1, dtype=np.int64)
    np.cumsum([s.numel for s in segs], out=off[1:])
    return off


def scaled_layout(segs: Sequence[Segment], divisor: int, ragged: bool = True) -> List[Segment]:
    """The same bucket structure with every tensor shrunk by `divisor` (for sizes the oracle
    finishes in seconds); `ragged` makes the sizes odd so segment starts lose their alignment."""
    out = []
    for i, s in enumerate(segs):
        m = max(1, s.numel // divisor)
        if ragged:
            m += (i * 7) % 5
        out.append(Segment(s.name, m))
    return out


def segment_params(n_seg: int, seed: int, alpha_range: Tuple[float, float], beta_range: Tuple[float, float],
                   log_alpha: bool) -> Tuple[np.ndarray, np.ndarray]:
    """Per-segment (alpha, beta): alpha log-uniform or uniform in alpha_range, beta uniform."""
    rng = np.random.Generator(np.random.Philox(seed))
    u = rng.random(n_seg)
    if log_alpha:
        alpha = np.exp(math.log(alpha_range[0]) + u * (math.log(alpha_range[1]) - math.log(alpha_range[0])))
    else:
        alpha = alpha_range[0] + u * (alpha_range[1] - alpha_range[0])
    beta = beta_range[0] + rng.random(n_seg) * (beta_range[1] - beta_range[0])
    return alpha, beta


def make_bucket(segs: Sequence[Segment], seed: int, device, dtype=None,
                alpha_range=(1e-5, 1e-3), beta_range=(0.5, 1.5), log_alpha=True):
    """Flat tensor holding every segment, segment s ~ GG(alpha_s, beta_s).
    Returns (flat tensor, offsets int64 ndarray, alpha ndarray, beta ndarray)."""
    dtype = dtype or torch.float32
    off = offsets_of(segs)
    alpha, beta = segment_params(len(segs), seed, alpha_range, beta_range, log_alpha)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    flat = torch.empty(int(off[-1]), dtype=dtype, device=device)
    for s, seg in enumerate(segs):
        flat[int(off[s]):int(off[s + 1])] = gg_torch(seg.numel, float(alpha[s]), float(beta[s]), gen, device,
                                                     dtype)
    return flat, off, alpha, beta


def make_tensor(shape, alpha: float, beta: float, seed: int, device, dtype=None,
                outlier_frac: float = 0.0, outlier_scale: float = 1.0) -> "torch.Tensor":
    """One GG tensor; optionally a fraction of uniformly chosen positions is multiplied by
    outlier_scale (activation outliers)."""
    dtype = dtype or torch.float32
    n = int(np.prod(shape))
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = gg_torch(n, alpha, beta, gen, device, torch.float32)
    if outlier_frac > 0.0:
        k = int(round(n * outlier_frac))
        pos = torch.randperm(n, generator=gen, device=device)[:k]
        x[pos] *= outlier_scale
    return x.to(dtype).reshape(shape)
