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


class deferred_weight_grads:
    """Context manager: DPLinear backward passes inside it only record (X, dY) of their layer; on exit all
    recorded layers go to the library in ONE flashdp_block_dp_grad call per (B, T, dtype) group, so that the
    per-block schedule applies (the aggregation of one layer running beside the contraction of the next)
    instead of one isolated call per layer.  The weights' .grad fields are filled (or added to) on exit.  The
    price is that X and dY of every recorded layer stay alive until then."""

    _active = None

    def __init__(self, schedule="auto"):
        self.schedule = schedule
        self.pending = []

    def __enter__(self):
        if deferred_weight_grads._active is not None:
            raise RuntimeError("deferred_weight_grads does not nest")
        deferred_weight_grads._active = self
        return self

    def __exit__(self, exc_type, exc, tb):
        deferred_weight_grads._active = None
        if exc_type is None:
            self.flush()
        self.pending = []
        return False

    def flush(self):
        groups = {}
        for rec in self.pending:
            groups.setdefault((rec["B"], rec["T"], rec["X"].dtype), []).append(rec)
        for (B, T, _), recs in groups.items():
            layers = []
            for r in recs:
                r["out"] = torch.empty(r["weight"].shape, dtype=torch.float32, device=r["X"].device)
                layers.append(dict(X=r["X"], dY=r["dY"], d_in=r["weight"].shape[1], d_out=r["weight"].shape[0], C=r["C"],
                                   sigma=r["sigma"], seed=r["seed"], layer=r["layer"], out_grad=r["out"], out_norms=r["norms"]))
            # layers of one group share the noise flag only if they agree; otherwise one call per flag value
            for flag in sorted({r["add_noise"] for r in recs}, reverse=True):
                sub = [L for L, r in zip(layers, recs) if r["add_noise"] == flag]
                F.flashdp_block_dp_grad_micro(sub, B, T, F.dtype_code(recs[0]["X"]), self.schedule, accumulate=False, add_noise=flag)
            for r in recs:
                if r["module"] is not None and r["module"].keep_fp32_grad:
                    m = r["module"]
                    m.grad_fp32 = r["out"].clone() if m.grad_fp32 is None else m.grad_fp32 + r["out"]
                g = r["out"].to(r["weight"].dtype)
                r["weight"].grad = g if r["weight"].grad is None else r["weight"].grad + g
        self.pending = []


class _DPLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, C, sigma, seed, layer, schedule, norms_out, add_noise, module):
        ctx.save_for_backward(x, weight)
        ctx.cfg = (float(C), float(sigma), int(seed), int(layer), schedule, norms_out, bool(add_noise), module)
        return torch.matmul(x, weight.t())

    @staticmethod
    def backward(ctx, dy):
        x, weight = ctx.saved_tensors
        C, sigma, seed, layer, schedule, norms_out, add_noise, module = ctx.cfg
        nothing = (None,) * 8
        d_out, d_in = weight.shape
        B = x.shape[0]
        xs = x.reshape(B, -1, d_in).contiguous()
        dys = dy.reshape(B, -1, d_out).contiguous()
        T = xs.shape[1]
        if xs.dtype != dys.dtype:
            dys = dys.to(xs.dtype)
        norms = norms_out if norms_out is not None else torch.empty((B,), dtype=torch.float32, device=x.device)
        grad_x = torch.matmul(dy, weight) if ctx.needs_input_grad[0] else None
        pending = deferred_weight_grads._active
        if pending is not None:   # hand the layer to the per-block call made when the context exits
            pending.pending.append(dict(X=xs, dY=dys, B=B, T=T, weight=weight, C=C, sigma=sigma, seed=seed, layer=layer,
                                        norms=norms, add_noise=add_noise, module=module))
            return (grad_x, None) + nothing
        grad_w = torch.empty((d_out, d_in), dtype=torch.float32, device=x.device)
        L = [dict(X=xs, dY=dys, d_in=d_in, d_out=d_out, C=C, sigma=sigma, seed=seed, layer=layer,
                  out_grad=grad_w, out_norms=norms)]
        F.flashdp_block_dp_grad_micro(L, B, T, F.dtype_code(xs), schedule, accumulate=False, add_noise=add_noise)
        if module is not None and module.keep_fp32_grad:
            module.grad_fp32 = grad_w.clone() if module.grad_fp32 is None else module.grad_fp32 + grad_w
        return (grad_x, grad_w.to(weight.dtype)) + nothing


class DPLinear(torch.nn.Module):
    """y = x W^T (no bias: the paper's path covers linear weights only).  After backward(), weight.grad holds (torch
    adds across backward calls) sum_i clip(G_i) + sigma*C*z, and last_norms the per-sample norms.

    Noise and steps.  The Philox field is keyed by (seed, step, layer): `step` is folded into the seed, and with
    auto_step (the default) it advances by itself at every forward pass whose backward adds noise, so that two
    optimizer steps never receive the same field - the Gaussian mechanism of Algorithm 1 would be void otherwise
    (the difference of two updates would be noise-free).  last_seed is the seed the last forward pass used.
    Gradient accumulation over micro-batches (Appendix D.1): set add_noise = False for all micro-batches of a step but
    the last; every micro-batch is clipped per sample, torch sums the clipped sums in weight.grad, and the noise goes
    in once, with the last micro-batch (the step then advances once, too).
    weight.grad has the parameter's dtype; with keep_fp32_grad the unrounded fp32 sum is kept in grad_fp32 as well
    (the caller clears it with zero_fp32_grad())."""

    def __init__(self, d_in: int, d_out: int, C: float = 1.0, sigma: float = 1.0, seed: int = 0, layer: int = 0,
                 schedule="auto", dtype=torch.bfloat16, device="cuda", auto_step: bool = True, keep_fp32_grad: bool = False):
        super().__init__()
        self.weight = torch.nn.Parameter(torch.empty(d_out, d_in, dtype=dtype, device=device))
        torch.nn.init.normal_(self.weight, std=d_in ** -0.5)
        self.C, self.sigma, self.seed, self.layer, self.schedule = C, sigma, seed, layer, schedule
        self.step = 0
        self.auto_step = auto_step
        self.add_noise = True
        self.keep_fp32_grad = keep_fp32_grad
        self.grad_fp32 = None
        self.last_norms = None
        self.last_seed = None

    def noise_seed(self) -> int:
        return (self.seed + (self.step << 32)) & 0xFFFFFFFFFFFFFFFF

    def zero_fp32_grad(self):
        self.grad_fp32 = None

    def forward(self, x):
        self.last_norms = torch.empty((x.shape[0],), dtype=torch.float32, device=x.device)
        self.last_seed = self.noise_seed()
        y = _DPLinearFn.apply(x, self.weight, self.C, self.sigma, self.last_seed, self.layer, self.schedule,
                              self.last_norms, self.add_noise, self)
        if self.auto_step and self.add_noise and torch.is_grad_enabled():
            self.step += 1
        return y
