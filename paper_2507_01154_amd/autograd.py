"""Drop-in linear layer whose backward yields the clipped, noised weight gradient (the paper's delivery
vehicle, Section 4.2: operators with trainable parameters are wrapped in an autograd function).

Only glue lives here.  The weight gradient - the whole path of Algorithm 1 - comes from the HIP library
through flashdp_block_dp_grad; the two adjacent steps of a training step that are not part of the path
(the forward product Y = X W^T and the input gradient dX = dY W) are plain GEMMs left to torch.matmul.

The loss must be a SUM over samples (not a mean), so that dY[i] is sample i's own output gradient; the
batch dimension is the first one and everything between it and the feature dimension counts as tokens.
"""
from __future__ import annotations

import torch

from . import binding as F


class _DPLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, C, sigma, seed, layer, schedule, norms_out):
        ctx.save_for_backward(x, weight)
        ctx.cfg = (float(C), float(sigma), int(seed), int(layer), schedule, norms_out)
        return torch.matmul(x, weight.t())

    @staticmethod
    def backward(ctx, dy):
        x, weight = ctx.saved_tensors
        C, sigma, seed, layer, schedule, norms_out = ctx.cfg
        d_out, d_in = weight.shape
        B = x.shape[0]
        xs = x.reshape(B, -1, d_in).contiguous()
        dys = dy.reshape(B, -1, d_out).contiguous()
        T = xs.shape[1]
        if xs.dtype != dys.dtype:
            dys = dys.to(xs.dtype)
        grad_w = torch.empty((d_out, d_in), dtype=torch.float32, device=x.device)
        norms = norms_out if norms_out is not None else torch.empty((B,), dtype=torch.float32, device=x.device)
        L = [dict(X=xs, dY=dys, d_in=d_in, d_out=d_out, C=C, sigma=sigma, seed=seed, layer=layer,
                  out_grad=grad_w, out_norms=norms)]
        F.flashdp_block_dp_grad(L, B, T, F.dtype_code(xs), schedule)
        grad_x = torch.matmul(dy, weight) if ctx.needs_input_grad[0] else None
        return grad_x, grad_w.to(weight.dtype), None, None, None, None, None, None


class DPLinear(torch.nn.Module):
    """y = x W^T (no bias: the paper's path covers linear weights only).  After backward(), weight.grad is
    sum_i clip(G_i) + sigma*C*z and last_norms holds the per-sample norms.  `step` is folded into the Philox
    seed so that the noise differs from one optimizer step to the next; the caller advances it."""

    def __init__(self, d_in: int, d_out: int, C: float = 1.0, sigma: float = 1.0, seed: int = 0, layer: int = 0,
                 schedule="auto", dtype=torch.bfloat16, device="cuda"):
        super().__init__()
        self.weight = torch.nn.Parameter(torch.empty(d_out, d_in, dtype=dtype, device=device))
        torch.nn.init.normal_(self.weight, std=d_in ** -0.5)
        self.C, self.sigma, self.seed, self.layer, self.schedule = C, sigma, seed, layer, schedule
        self.step = 0
        self.last_norms = None

    def noise_seed(self) -> int:
        return (self.seed + (self.step << 32)) & 0xFFFFFFFFFFFFFFFF

    def forward(self, x):
        self.last_norms = torch.empty((x.shape[0],), dtype=torch.float32, device=x.device)
        return _DPLinearFn.apply(x, self.weight, self.C, self.sigma, self.noise_seed(), self.layer, self.schedule,
                                 self.last_norms)
