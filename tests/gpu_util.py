"""Helpers shared by the GPU parity tests: stored numpy values -> device buffers, one library call
through the C ABI, and the error measures the tolerances are written in."""
import os

import numpy as np
import torch

import paper_2507_01154_amd as F

DEV = "cuda:0"


def to_device(a: np.ndarray) -> torch.Tensor:
    """uint16 arrays are bfloat16 bit patterns; float16 / float32 arrays are taken as they are."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    d = np.linalg.norm(got.astype(np.float64) - want)
    n = np.linalg.norm(want)
    return float(d / n) if n > 0 else float(d)


def oracle_signal_and_bound(X, dY, C):
    """The sigma = 0 result of the oracle composed from its own stage functions, sample by sample, together with
    bound[e] = sum_i c_i |G_i[e]|: the magnitude the element-wise tolerance is scaled by (out[e] itself can be small
    through cancellation between samples while each term, and hence each term's rounding error, is not).
    Returns (out [D,P] fp64, norms [B] fp64, bound [D,P] fp64); out and norms are bit-identical to
    O.linear_dp_grad(X, dY, C, 0, ...) (checked in the CPU suite)."""
    from oracle import flashdp_oracle as O
    out = bound = None
    norms = np.zeros(X.shape[0])
    for i in range(X.shape[0]):
        G = O.per_sample_gradient(X[i], dY[i])
        norms[i] = O.frobenius_norm(G)
        G *= O.clip_factor(norms[i], float(C))
        out = G.copy() if out is None else out + G
        np.abs(G, out=G)
        bound = G if bound is None else bound + G
    return out, norms, bound


def elementwise_excess(got: np.ndarray, want: np.ndarray, bound: np.ndarray, parked_16bit: bool):
    """Element-wise check of the sigma = 0 signal.  Allowed |got - want| per element:
      fp32 accumulation over T products and B samples:        1e-4 * rms(bound)   (every path)
      plus, when the per-sample tile is parked as bfloat16:   2^-8 * bound[e]     (one rounding to 8 significant bits per term).
    Returns (worst ratio err / allowed, flat index of the worst element); <= 1 passes."""
    err = np.abs(got.astype(np.float64) - want)
    allowed = 1e-4 * float(np.sqrt(np.mean(np.square(bound))))
    allowed = allowed + (2.0 ** -8) * bound if parked_16bit else np.full_like(bound, allowed)
    ratio = err / allowed
    k = int(np.argmax(ratio))
    return float(ratio.reshape(-1)[k]), k


class env:
    """Sets environment variables for the duration of a with-block (with FLASHDP_DEBUG_ENV=1, which
    conftest.py sets, the library reads FLASHDP_TILE / FLASHDP_SCHEDULE at every call)."""

    def __init__(self, **kv):
        self.kv = {k: v for k, v in kv.items() if v is not None}

    def __enter__(self):
        self.old = {k: os.environ.get(k) for k in self.kv}
        os.environ.update({k: str(v) for k, v in self.kv.items()})

    def __exit__(self, *a):
        for k, v in self.old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


def run_layer(X: np.ndarray, dY: np.ndarray, C, sigma, seed, layer=0, schedule="auto", workspace=None, tile=None):
    """One flashdp_block_dp_grad call for a single layer; returns (out [D,P] fp32, norms [B] fp32, schedule used)."""
    B, T, P = X.shape
    D = dY.shape[2]
    dX, ddY = to_device(X), to_device(dY)
    out = torch.full((D, P), float("nan"), device=DEV, dtype=torch.float32)      # poisoned: must be overwritten
    norms = torch.full((B,), float("nan"), device=DEV, dtype=torch.float32)
    L = dict(X=dX, dY=ddY, d_in=P, d_out=D, C=C, sigma=sigma, seed=seed, layer=layer, out_grad=out, out_norms=norms)
    with env(FLASHDP_TILE=tile):
        F.flashdp_block_dp_grad([L], B, T, F.dtype_code(dX), schedule, workspace)
    torch.cuda.synchronize()
    return out.cpu().numpy(), norms.cpu().numpy(), F.flashdp_last_schedule()
