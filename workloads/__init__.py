"""Seeded synthetic inputs for the per-layer DP weight-gradient path.

This module only *draws numbers*: it holds none of the method's arithmetic (no
contraction, norm, clip factor or noise).  Both the CPU oracle's tests and the HIP
path's tests/benchmark take their inputs from here, so that the two are compared
on identical stored values.

Each workload mirrors one of the benchmark configurations: linear layers of GPT-2
(T = 1024) and Llama (T = 2048) shape, the models the paper trains (Section 5.1,
"Experimental Setup").  The paper's datasets are not used; activations X are
standard normal and output gradients dY are normal with a small variance times a
per-sample scale, which puts every per-sample gradient norm above the clipping
threshold, the regime DP training lives in.

Storage formats handed out:
  * "bf16": numpy uint16 arrays holding bfloat16 bit patterns (round-to-nearest-even
    from the float32 draw);
  * "f16": numpy float16 arrays (round-to-nearest-even from the float32 draw);
  * "fp32": numpy float32 arrays.
The consumer decides how to widen them; nothing here interprets them further.

Streams: every (workload, layer, sample, tensor) has its own numpy Generator seeded
from the tuple, so any slice can be regenerated alone (the benchmark's CPU leg
regenerates one sample without building the whole batch).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

_TENSOR_X = 0
_TENSOR_DY = 1
_TENSOR_SCALE = 2


@dataclass(frozen=True)
class LayerSpec:
    name: str
    d_in: int   # P
    d_out: int  # D


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "bf16", "f16" or "fp32"
    B: int
    T: int
    layers: Tuple[LayerSpec, ...]
    dy_variance: float    # variance of dY before the per-sample scale
    scale_rule: str       # "pow10" (10^(i-2)) or "loguniform" (10^U(-1,1))
    C: float
    sigma: float
    data_seed: int
    noise_seed: int       # layer l uses noise_seed + l and layer index l

    def layer_seed(self, l: int) -> int:
        return self.noise_seed + l

    def flops(self) -> int:
        """Algorithmic FLOPs of one pass: one contraction per layer."""
        return sum(2 * self.B * self.T * s.d_in * s.d_out for s in self.layers)


def _llama13b_block() -> Tuple[LayerSpec, ...]:
    h, f = 5120, 13824
    return (
        LayerSpec("q_proj", h, h), LayerSpec("k_proj", h, h),
        LayerSpec("v_proj", h, h), LayerSpec("o_proj", h, h),
        LayerSpec("gate_proj", h, f), LayerSpec("up_proj", h, f),
        LayerSpec("down_proj", f, h),
    )


WORKLOADS: Dict[str, Workload] = {
    # configuration 1: tiny fp32 layer; sigma is 0 or 1 depending on the check.
    "tiny_fp32": Workload("tiny_fp32", "fp32", 4, 16, (LayerSpec("linear", 32, 32),),
                          1.0, "pow10", 1.0, 1.0, 0, 1),
    # configuration 2: GPT-2-small MLP up-projection.
    "gpt2_small_mlp_up": Workload("gpt2_small_mlp_up", "bf16", 8, 1024,
                                  (LayerSpec("c_fc", 768, 3072),),
                                  1e-3, "loguniform", 1.0, 1.0, 2, 1),
    # configuration 3: Llama-7B attention q_proj.
    "llama7b_q_proj": Workload("llama7b_q_proj", "bf16", 4, 2048,
                               (LayerSpec("q_proj", 4096, 4096),),
                               1e-4, "loguniform", 1.0, 0.8, 3, 1),
    # the precision variants of the mixed-precision experiment (Appendix D.2) on the configuration-3 layer
    "llama7b_q_proj_fp32": Workload("llama7b_q_proj_fp32", "fp32", 4, 2048,
                                    (LayerSpec("q_proj", 4096, 4096),),
                                    1e-4, "loguniform", 1.0, 0.8, 3, 1),
    "llama7b_q_proj_f16": Workload("llama7b_q_proj_f16", "f16", 4, 2048,
                                   (LayerSpec("q_proj", 4096, 4096),),
                                   1e-4, "loguniform", 1.0, 0.8, 3, 1),
    # configuration 4: Llama-13B MLP up_proj.
    "llama13b_up_proj": Workload("llama13b_up_proj", "bf16", 4, 2048,
                                 (LayerSpec("up_proj", 5120, 13824),),
                                 1e-4, "loguniform", 1.0, 1.0, 4, 1),
    # configuration 5: full Llama-13B decoder block, 7 linears, independent tensors.
    "llama13b_block": Workload("llama13b_block", "bf16", 8, 2048, _llama13b_block(),
                               1e-4, "loguniform", 1.0, 1.0, 5, 1),
}


def float32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.

    Finite inputs only (the generators never produce NaN/Inf)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def sample_scales(w: Workload, layer: int) -> np.ndarray:
    """Per-sample multiplier of dY for one layer, float64[B]."""
    if w.scale_rule == "pow10":
        return 10.0 ** (np.arange(w.B, dtype=np.float64) - 2.0)
    if w.scale_rule == "loguniform":
        rng = np.random.default_rng([w.data_seed, layer, 0, _TENSOR_SCALE])
        return 10.0 ** rng.uniform(-1.0, 1.0, size=w.B)
    raise ValueError(w.scale_rule)


def _store(a32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return float32_to_bf16_bits(a32)
    if dtype == "f16":
        return a32.astype(np.float16)
    if dtype == "fp32":
        return a32
    raise ValueError(dtype)


def make_sample(w: Workload, layer: int, i: int, T: int | None = None):
    """(X_i [T,P], dY_i [T,D]) of one sample in the workload's storage format.

    T may be given smaller than the workload's to take a prefix of the tokens of a
    (differently seeded) shorter sequence; default is the workload's T."""
    spec = w.layers[layer]
    T = w.T if T is None else T
    rx = np.random.default_rng([w.data_seed, layer, i, _TENSOR_X])
    ry = np.random.default_rng([w.data_seed, layer, i, _TENSOR_DY])
    x = rx.standard_normal((T, spec.d_in), dtype=np.float32)
    dy = ry.standard_normal((T, spec.d_out), dtype=np.float32)
    s = np.float32(np.sqrt(w.dy_variance) * sample_scales(w, layer)[i])
    dy *= s
    return _store(x, w.dtype), _store(dy, w.dtype)


def make_layer(w: Workload, layer: int, threads: int = 8):
    """(X [B,T,P], dY [B,T,D]) for one layer, storage format per w.dtype."""
    spec = w.layers[layer]
    np_dt = {"bf16": np.uint16, "f16": np.float16, "fp32": np.float32}[w.dtype]
    X = np.empty((w.B, w.T, spec.d_in), dtype=np_dt)
    dY = np.empty((w.B, w.T, spec.d_out), dtype=np_dt)

    def fill(i):
        X[i], dY[i] = make_sample(w, layer, i)

    if threads > 1 and w.B > 1 and X.size + dY.size > (1 << 22):
        with ThreadPoolExecutor(max_workers=min(threads, w.B)) as ex:
            list(ex.map(fill, range(w.B)))
    else:
        for i in range(w.B):
            fill(i)
    return X, dY


def scaled_down(w: Workload, B: int | None = None, T: int | None = None,
                dims: List[Tuple[int, int]] | None = None, name: str | None = None) -> Workload:
    """A smaller workload with the same value recipe (for parity cases the oracle
    finishes in seconds).  dims = [(d_in, d_out), ...] replaces the layer shapes."""
    layers = w.layers
    if dims is not None:
        layers = tuple(LayerSpec(f"l{k}", di, do) for k, (di, do) in enumerate(dims))
    return Workload(name or (w.name + "_small"), w.dtype, B or w.B, T or w.T, layers,
                    w.dy_variance, w.scale_rule, w.C, w.sigma, w.data_seed, w.noise_seed)


def make_layer_device(w: Workload, layer: int, device: str = "cuda:0"):
    """Same recipe as make_layer, drawn on the device with torch's seeded generator (another stream of
    numbers, same distributions): for the benchmark, where 3 GB of host draws would dominate the run.
    Returns torch tensors (X [B,T,P], dY [B,T,D]) of the workload's dtype."""
    import torch

    spec = w.layers[layer]
    dt = {"bf16": torch.bfloat16, "f16": torch.float16, "fp32": torch.float32}[w.dtype]
    g = torch.Generator(device=device)
    g.manual_seed((w.data_seed << 8) + layer)
    scales = torch.tensor(np.sqrt(w.dy_variance) * sample_scales(w, layer), dtype=torch.float32, device=device)
    X = torch.empty((w.B, w.T, spec.d_in), dtype=dt, device=device)
    dY = torch.empty((w.B, w.T, spec.d_out), dtype=dt, device=device)
    for i in range(w.B):       # sample by sample: the fp32 draw is transient
        X[i] = torch.randn((w.T, spec.d_in), generator=g, device=device, dtype=torch.float32).to(dt)
        dY[i] = (torch.randn((w.T, spec.d_out), generator=g, device=device, dtype=torch.float32) * scales[i]).to(dt)
    return X, dY
