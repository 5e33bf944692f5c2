"""Thin PyTorch glue over libgg for the paper's three uses of the pass: GG initialisation (Sec. 4.1,
Eq. 5), the activation rate term of ACT (Sec. 4.2) as a differentiable op, and the GCT update
(Sec. 4.3, Algorithm 2).  Every numeric step runs in the library's kernels; torch only carries
tensors, the autograd graph and the stream."""
from __future__ import annotations

from typing import Iterable, Optional, Tuple

import torch

from . import binding as B


def gg_init_(params: Iterable[Tuple[torch.Tensor, int]], shape: float, xi: float = 1.0, seed: int = 0) -> None:
    """GG initialisation: fills each (weight, fan_in) in place with GG(0, alpha, shape) variates,
    alpha = sqrt(xi/fan_in * Gamma(1/shape)/Gamma(3/shape)) (Eq. 5; shape 2 is He initialisation).
    Tensor i draws from generator stream i of `seed`, so the result does not depend on tensor sizes
    or launch shapes."""
    for i, (w, fan_in) in enumerate(params):
        if not w.is_contiguous():
            raise ValueError("gg_init_ needs contiguous parameters")
        alpha = B.gg_init_alpha(fan_in, shape, xi)
        B.gg_sample(w.numel(), alpha, shape, seed, stream_id=i, out=w.view(-1))


class EGRate(torch.autograd.Function):
    """R(A) of Sec. 4.2: mean order-k Exp-Golomb length of the activations quantised with step
    `delta` (2^-n in the paper).  Backward is the straight-through gradient
    4 (1/delta) / (N ln 2) * sign(a) / (Map(floor(a/delta)) + 2^k)."""

    @staticmethod
    def forward(ctx, a: torch.Tensor, delta: float, eg_k: int = 0):
        flat = a.contiguous().view(-1)
        ws = B.Workspace(flat.numel(), 1, device=flat.device)
        rec, _, _ = B.gg_quantize_rate(flat, delta, ws, eg_k=eg_k)
        ctx.save_for_backward(flat)
        ctx.delta, ctx.eg_k, ctx.shape, ctx.dtype = delta, eg_k, a.shape, a.dtype
        bits = rec[:8].view(torch.int64)            # gg_rate_t.eg_bits, still on the device
        return (bits.to(torch.float64) / flat.numel()).to(torch.float32).reshape(())

    @staticmethod
    def backward(ctx, grad_out):
        (flat,) = ctx.saved_tensors
        # the incoming scalar (lambda_act of J = D + lambda_act R) goes into the kernel as its `scale`
        # argument: reading it costs one device-to-host copy of four bytes, no torch arithmetic
        g = B.gg_rate_grad(flat, ctx.delta, eg_k=ctx.eg_k, scale=float(grad_out))
        return g.to(ctx.dtype).reshape(ctx.shape), None, None


def eg_rate(a: torch.Tensor, delta: float, eg_k: int = 0) -> torch.Tensor:
    return EGRate.apply(a, delta, eg_k)


class GCTState:
    """Per-bucket state of Algorithm 2: the previous equivalent gradient, the step counter and the
    decaying multiplier lambda_tau.  `step` applies the update to a flat fp32 parameter bucket."""

    def __init__(self, n: int, offsets, eta: float, lam: float, eps: float = 1e-8, decay: float = 0.8,
                 delta_div: float = 16.0, eg_k: int = 0, device="cuda"):
        self.offsets, self.eta, self.lam, self.eps, self.decay = offsets, eta, lam, eps, decay
        self.delta_div, self.eg_k = delta_div, eg_k
        self.ghat_prev = torch.zeros(n, dtype=torch.float32, device=device)
        self.ws = B.Workspace(n, len(offsets) - 1, device=device)
        self.t = 1

    def step(self, w: torch.Tensor, g: torch.Tensor) -> dict:
        """One batch: fit and rate of the gradient bucket (the monitored EG length), then the update."""
        res = B.gg_fused_segmented(g, self.offsets, self.ws, delta_div=self.delta_div, eg_k=self.eg_k)
        delta = B.gg_delta_from_fit(res["fit"], len(self.offsets) - 1, self.delta_div)
        B.gg_gct_update_segmented(w, g, self.ghat_prev, self.offsets, delta, self.eta, self.lam, self.eps, self.ws,
                                  eg_k=self.eg_k, first_step=self.t == 1)
        self.t += 1
        return res

    def end_epoch(self) -> None:
        self.lam *= self.decay      # constraint decay lambda <- alpha * lambda
