"""CPU oracle for the per-layer DP weight gradient of a linear layer (FlashDP).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that the
HIP library is checked against.  Nothing in the product path may import it; it
imports nothing from the product either.  Allowed callers: tests/, the smoke check
and the benchmark's cpu_baseline leg.

What it computes (the paper's explicit four-stage DP-SGD flow for one linear layer,
Appendix B.2 "Explicit DP-SGD Workflow", with the formulas of Algorithm 1,
"FlashDP with Block-wise All-Reduce"; the fused method reaches exactly this result,
as the utility table of Appendix D.3 asserts, so the oracle is the plain definition):

  stage 1   G_i[d][p] = sum_t dY[i][t][d] * X[i][t][p]          (Eq. per-sample-grad, Format 2)
  stage 2   n_i       = sqrt(sum_{d,p} G_i[d][p]^2)             (Section 3, Stage 2; Alg. 1 "Intra/Inter-block Reduce")
  stage 3   c_i       = 1 / max(1, n_i / C)                     (Alg. 1 clip step; Appendix B.2 Stage 3)
  stage 4   out[d][p] = sum_i c_i G_i[d][p] + sigma*C*z[d*P+p]  (Alg. 1 noise/aggregate step; Stage 4)

Readings where the paper is silent or inconsistent (all listed in the design notes):
  * batch SUM, no 1/B (Alg. 1 and Stage 4 print a sum; Appendix A.1 prints a mean);
  * the square under the root in Stage 2 of Appendix B.2 is missing in print; Section 3
    and Alg. 1 have it;
  * max-form of the clip factor, so a zero gradient gives c_i = 1 and no division by zero;
  * noise is added once per output element of the layer, with std sigma*C;
  * the paper names no random generator.  z is a counter-based field: Philox4x32-10
    (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11)
    with key = (seed mod 2^32, seed div 2^32) and counter = (g mod 2^32, g div 2^32, layer, 0),
    g = e div 4, e = d*P + p; the four output words r0..r3 serve elements 4g..4g+3 through
    Box-Muller on 24-bit uniforms u(r) = ((r div 256) + 1/2) / 2^24:
        z0 = rho(r0) cos(2 pi u(r1)), z1 = rho(r0) sin(2 pi u(r1)),
        z2 = rho(r2) cos(2 pi u(r3)), z3 = rho(r2) sin(2 pi u(r3)),  rho(r) = sqrt(-2 ln u(r)).

Inputs are the exact stored values (bfloat16 bit patterns or float32) widened to fp64.
All floating point below is fp64; the contraction of stage 1 is one library matmul per
sample (no blocking, fusion or reordering of the definition).

Pins (tests/test_oracle_*.py, all CPU): Philox known-answer vectors from the SC'11
reference distribution; a hand-worked 2x2 example; brute-force loops on tiny integer
inputs; the ghost-norm identity as an independent route to n_i; rank-1 and identity-X
closed forms; clip invariants; normality of the noise field (moments, KS) and its
independence from everything but (seed, layer, e).
Parity unpinned: nothing in this file.  (Bias gradients are outside the path.)
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------------
# stored value -> fp64
# ----------------------------------------------------------------------------------

def widen(a: np.ndarray) -> np.ndarray:
    """Exact fp64 value of stored inputs: uint16 = bfloat16 bit patterns, float32/64 as is."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if a.dtype in (np.float32, np.float64):
        return a.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {a.dtype}")


# ----------------------------------------------------------------------------------
# Philox4x32-10 (SC'11), vectorised over counters
# ----------------------------------------------------------------------------------

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(counter: np.ndarray, key) -> np.ndarray:
    """counter: uint32 array [..., 4]; key: two uint32 words.  Returns uint32 [..., 4]."""
    c = np.asarray(counter, dtype=np.uint32)
    c0 = c[..., 0].astype(np.uint64)
    c1 = c[..., 1].astype(np.uint64)
    c2 = c[..., 2].astype(np.uint64)
    c3 = c[..., 3].astype(np.uint64)
    k0 = int(key[0]) & 0xFFFFFFFF
    k1 = int(key[1]) & 0xFFFFFFFF
    for rnd in range(10):
        if rnd > 0:  # the key schedule: add the Weyl constants before every round but the first
            k0 = (k0 + _W0) & 0xFFFFFFFF
            k1 = (k1 + _W1) & 0xFFFFFFFF
        p0 = _M0 * c0  # 32x32 -> 64 bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0)), lo1, (hi0 ^ c3 ^ np.uint64(k1)), lo0
    out = np.empty(c.shape, dtype=np.uint32)
    out[..., 0] = c0
    out[..., 1] = c1
    out[..., 2] = c2
    out[..., 3] = c3
    return out


# ----------------------------------------------------------------------------------
# Gaussian noise field z(seed, layer, e)
# ----------------------------------------------------------------------------------

def uniform24(r: np.ndarray) -> np.ndarray:
    """u(r) = ((r div 2^8) + 1/2) / 2^24, strictly inside (0, 1)."""
    return ((np.asarray(r, dtype=np.uint32) >> np.uint32(8)).astype(np.float64) + 0.5) / 16777216.0


def gaussians_from_words(r: np.ndarray) -> np.ndarray:
    """r: uint32 [..., 4] -> z: float64 [..., 4] by two Box-Muller pairs."""
    u0, u1, u2, u3 = (uniform24(r[..., k]) for k in range(4))
    rho_a = np.sqrt(-2.0 * np.log(u0))
    rho_b = np.sqrt(-2.0 * np.log(u2))
    z = np.empty(r.shape, dtype=np.float64)
    z[..., 0] = rho_a * np.cos(2.0 * np.pi * u1)
    z[..., 1] = rho_a * np.sin(2.0 * np.pi * u1)
    z[..., 2] = rho_b * np.cos(2.0 * np.pi * u3)
    z[..., 3] = rho_b * np.sin(2.0 * np.pi * u3)
    return z


def _group_counters(g: np.ndarray, layer: int) -> np.ndarray:
    g = np.asarray(g, dtype=np.uint64)
    ctr = np.empty(g.shape + (4,), dtype=np.uint32)
    ctr[..., 0] = (g & _MASK32).astype(np.uint32)
    ctr[..., 1] = (g >> _SH32).astype(np.uint32)
    ctr[..., 2] = np.uint32(int(layer) & 0xFFFFFFFF)
    ctr[..., 3] = 0
    return ctr


def _key(seed: int):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return (seed & 0xFFFFFFFF, seed >> 32)


def noise_at(seed: int, layer: int, e: np.ndarray) -> np.ndarray:
    """z at the given flat element indices e (any shape), fp64."""
    e = np.asarray(e, dtype=np.uint64)
    z4 = gaussians_from_words(philox4x32_10(_group_counters(e >> np.uint64(2), layer), _key(seed)))
    lane = (e & np.uint64(3)).astype(np.int64)
    return np.take_along_axis(z4, lane[..., None], axis=-1)[..., 0]


def noise_field(seed: int, layer: int, n: int, chunk_groups: int = 1 << 21) -> np.ndarray:
    """z[0..n), fp64; element e uses group e div 4, slot e mod 4."""
    n = int(n)
    out = np.empty(n, dtype=np.float64)
    n_groups = (n + 3) // 4
    for g0 in range(0, n_groups, chunk_groups):
        g1 = min(n_groups, g0 + chunk_groups)
        g = np.arange(g0, g1, dtype=np.uint64)
        z4 = gaussians_from_words(philox4x32_10(_group_counters(g, layer), _key(seed))).reshape(-1)
        e0, e1 = 4 * g0, min(n, 4 * g1)
        out[e0:e1] = z4[: e1 - e0]
    return out


# ----------------------------------------------------------------------------------
# stages 1-4
# ----------------------------------------------------------------------------------

def per_sample_gradient(X_i: np.ndarray, dY_i: np.ndarray) -> np.ndarray:
    """Stage 1 for one sample: G_i = dY_i^T X_i, [D, P] fp64.  X_i [T,P], dY_i [T,D] stored values."""
    return widen(dY_i).T @ widen(X_i)


def frobenius_norm(G_i: np.ndarray) -> float:
    """Stage 2: sqrt of the sum of squares over both feature axes."""
    return float(np.sqrt(np.sum(np.square(G_i))))


def clip_factor(n_i: float, C: float) -> float:
    """Stage 3: 1 / max(1, n_i / C)."""
    return 1.0 / max(1.0, n_i / C)


def linear_dp_grad(X, dY, C: float, sigma: float, seed: int, layer: int = 0):
    """Stages 1-4 for one layer.

    X [B,T,P], dY [B,T,D] stored values (uint16 bf16 bits or float32).
    Returns (out [D,P] fp64, norms [B] fp64 = pre-clip n_i)."""
    X = np.asarray(X)
    dY = np.asarray(dY)
    B, T, P = X.shape
    assert dY.shape[:2] == (B, T)
    D = dY.shape[2]
    C = float(C)
    out = np.zeros((D, P), dtype=np.float64)
    norms = np.zeros(B, dtype=np.float64)
    for i in range(B):
        G_i = per_sample_gradient(X[i], dY[i])
        norms[i] = frobenius_norm(G_i)
        out += clip_factor(norms[i], C) * G_i
    if sigma != 0.0:
        out += (float(sigma) * C) * noise_field(seed, layer, D * P).reshape(D, P)
    return out, norms


def accumulated_dp_grad(micro_batches, C: float, sigma: float, seed: int, layer: int = 0):
    """Gradient accumulation over micro-batches (the setting of the paper's micro-batch table, Appendix D.1;
    the paper does not write the rule out).  Reading: every sample is clipped by its own norm as in
    stages 1-3, the clipped gradients of all micro-batches are summed, and the noise of stage 4 is added
    once for the accumulated batch.

    micro_batches: iterable of (X [b,T,P], dY [b,T,D]).  Returns (out [D,P], list of norms per micro-batch)."""
    out = None
    all_norms = []
    for X, dY in micro_batches:
        part, norms = linear_dp_grad(X, dY, C, 0.0, seed, layer)     # stages 1-3 and the clipped sum, no noise
        out = part if out is None else out + part
        all_norms.append(norms)
    if sigma != 0.0:
        D, P = out.shape
        out = out + (float(sigma) * float(C)) * noise_field(seed, layer, D * P).reshape(D, P)
    return out, all_norms


def block_dp_grad(layers):
    """Per-layer clipping over several linears (Algorithm "Per-Layer Gradient Processing",
    Appendix A.1): each layer is processed on its own with its own (C, sigma, seed, layer).

    layers: iterable of dicts with keys X, dY, C, sigma, seed, layer.
    Returns a list of (out, norms)."""
    return [linear_dp_grad(L["X"], L["dY"], L["C"], L["sigma"], L["seed"], L["layer"]) for L in layers]
