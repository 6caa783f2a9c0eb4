"""Pins for stages 1-4 of the oracle: hand-worked values, brute force, closed forms,
an independent route to the norms, and the invariants of clipping."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import flashdp_oracle as O
import workloads as W


def _read_golden(path):
    d = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            d[k] = np.array([float(x) for x in v])
    return d


def test_widen_bf16_bit_patterns():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x3DCD, 0x7F7F, 0x0080], dtype=np.uint16)
    v = O.widen(bits)
    assert v[0] == 1.0 and v[1] == -2.0 and v[2] == 0.0 and v[3] == 0.0 and math.copysign(1, v[3]) == -1
    assert v[4] == (1 + 0x4D / 128.0) * 2.0 ** (0x7B - 127)       # 0x3DCD: exponent 0x7B, mantissa 0x4D
    assert v[5] == (2 - 2.0 ** -7) * 2.0 ** 127
    assert v[6] == 2.0 ** -126
    f = np.array([0.1, -3.5], dtype=np.float32)
    assert np.array_equal(O.widen(f), f.astype(np.float64))


def test_hand_worked_2x2(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "worked_2x2.txt"))
    X = np.stack([g["X0"].reshape(2, 2), g["X1"].reshape(2, 2)]).astype(np.float32)
    dY = np.stack([g["dY0"].reshape(2, 2), g["dY1"].reshape(2, 2)]).astype(np.float32)
    assert np.array_equal(O.per_sample_gradient(X[0], dY[0]), g["G0"].reshape(2, 2))
    assert np.array_equal(O.per_sample_gradient(X[1], dY[1]), g["G1"].reshape(2, 2))
    out, norms = O.linear_dp_grad(X, dY, C=g["C"][0], sigma=0.0, seed=0)
    assert np.allclose(norms ** 2, g["normsq"], rtol=1e-14)
    assert np.allclose(out.reshape(-1), g["out"], rtol=1e-14, atol=0)
    # the same values stored as bf16 (small integers are exact in bf16)
    out_b, norms_b = O.linear_dp_grad(W.float32_to_bf16_bits(X), W.float32_to_bf16_bits(dY), g["C"][0], 0.0, 0)
    assert np.array_equal(out_b, out) and np.array_equal(norms_b, norms)


def _brute(X, dY, C):
    """Definition by loops, outermost over output elements (a different order from the oracle)."""
    B, T, P = X.shape
    D = dY.shape[2]
    G = [[[0.0] * P for _ in range(D)] for _ in range(B)]
    for p in range(P):
        for d in range(D):
            for i in range(B):
                s = 0.0
                for t in range(T):
                    s += float(dY[i][t][d]) * float(X[i][t][p])
                G[i][d][p] = s
    norms = []
    for i in range(B):
        s = 0.0
        for d in range(D):
            for p in range(P):
                s += G[i][d][p] ** 2
        norms.append(math.sqrt(s))
    out = [[0.0] * P for _ in range(D)]
    for i in range(B):
        c = min(1.0, C / norms[i]) if norms[i] > 0 else 1.0     # min-form of the clip (Appendix A.1)
        for d in range(D):
            for p in range(P):
                out[d][p] += c * G[i][d][p]
    return np.array(out), np.array(norms)


@pytest.mark.parametrize("shape", [(2, 3, 2, 2), (3, 5, 4, 3), (2, 1, 3, 5)])
def test_brute_force_small_integers(shape):
    B, T, P, D = shape
    rng = np.random.default_rng(sum(shape))
    X = rng.integers(-3, 4, size=(B, T, P)).astype(np.float32)
    dY = rng.integers(-3, 4, size=(B, T, D)).astype(np.float32)
    for C in (0.5, 6.0, 1e9):
        want, wn = _brute(X, dY, C)
        got, gn = O.linear_dp_grad(X, dY, C, 0.0, 0)
        assert got.shape == (D, P)
        assert np.allclose(gn, wn, rtol=1e-13)
        assert np.allclose(got, want, rtol=1e-13, atol=1e-13)


def test_brute_force_tiny_config_and_torch_second_opinion():
    w = W.WORKLOADS["tiny_fp32"]
    X, dY = W.make_layer(w, 0)
    out, norms = O.linear_dp_grad(X, dY, w.C, 0.0, w.noise_seed)
    want, wn = _brute(X, dY, w.C)
    assert np.allclose(norms, wn, rtol=1e-12) and np.allclose(out, want, rtol=1e-11, atol=1e-14)
    G = torch.einsum("btd,btp->bdp", torch.from_numpy(dY).double(), torch.from_numpy(X).double())
    n = G.flatten(1).norm(dim=1)
    ref = (G / torch.clamp(n / w.C, min=1.0)[:, None, None]).sum(0)
    assert np.allclose(norms, n.numpy(), rtol=1e-12)
    assert np.allclose(out, ref.numpy(), rtol=1e-11, atol=1e-14)
    # the configuration as written: every sample has a norm above C = 1 (printed for the record)
    print("tiny_fp32 realised norms:", norms)
    assert np.all(norms > 1.0)
    # companion case C = 20: samples 0,1 pass unclipped, 2,3 clip
    assert norms[0] < 20 and norms[1] < 20 and norms[2] > 20 and norms[3] > 20


def test_ghost_norm_identity_is_an_independent_route():
    # ||dY^T X||_F^2 = sum_{t,t'} (dy_t . dy_t') (x_t . x_t')   (the ghost-clipping identity cited in Section 2)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((3, 7, 6)).astype(np.float32)
    dY = rng.standard_normal((3, 7, 4)).astype(np.float32)
    _, norms = O.linear_dp_grad(X, dY, 1.0, 0.0, 0)
    for i in range(3):
        a = dY[i].astype(np.float64) @ dY[i].astype(np.float64).T
        b = X[i].astype(np.float64) @ X[i].astype(np.float64).T
        assert abs(norms[i] ** 2 - np.sum(a * b)) < 1e-10 * norms[i] ** 2


def test_closed_forms():
    rng = np.random.default_rng(11)
    # T = 1: rank one, ||G|| = ||dy|| ||x||
    X = rng.standard_normal((2, 1, 5)).astype(np.float32)
    dY = rng.standard_normal((2, 1, 3)).astype(np.float32)
    _, norms = O.linear_dp_grad(X, dY, 1.0, 0.0, 0)
    for i in range(2):
        want = np.linalg.norm(dY[i, 0].astype(np.float64)) * np.linalg.norm(X[i, 0].astype(np.float64))
        assert abs(norms[i] - want) < 1e-13 * want
    # X = [I_T | 0]: G = [dY^T | 0]  -> catches a transposed operand
    T, P, D = 3, 5, 4
    X = np.zeros((1, T, P), np.float32)
    X[0, :, :T] = np.eye(T)
    dY = rng.standard_normal((1, T, D)).astype(np.float32)
    G = O.per_sample_gradient(X[0], dY[0])
    assert G.shape == (D, P)
    assert np.array_equal(G[:, :T], dY[0].T.astype(np.float64)) and np.all(G[:, T:] == 0)
    # B = 1, clipped: ||out|| = C exactly (up to rounding)
    X = rng.standard_normal((1, 4, 6)).astype(np.float32)
    dY = 50 * rng.standard_normal((1, 4, 3)).astype(np.float32)
    out, norms = O.linear_dp_grad(X, dY, 0.25, 0.0, 0)
    assert norms[0] > 0.25 and abs(np.linalg.norm(out) - 0.25) < 1e-14
    # zero gradient: factor 1, no division by zero
    out, norms = O.linear_dp_grad(np.zeros((2, 3, 4), np.float32), np.ones((2, 3, 2), np.float32), 1.0, 0.0, 0)
    assert np.all(norms == 0) and np.all(out == 0) and np.all(np.isfinite(out))
    assert O.clip_factor(0.0, 1.0) == 1.0 and O.clip_factor(1.0, 1.0) == 1.0 and O.clip_factor(4.0, 1.0) == 0.25


def _rand(B, T, P, D, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((B, T, P)).astype(np.float32),
            (scale * rng.standard_normal((B, T, D))).astype(np.float32))


def test_invariants_of_clipping_and_aggregation():
    B, T, P, D = 4, 6, 5, 7
    X, dY = _rand(B, T, P, D, 3)
    dY *= np.array([0.01, 0.1, 1, 10], np.float32)[:, None, None]
    C = 1.0
    out, norms = O.linear_dp_grad(X, dY, C, 0.0, 0)
    c = np.array([O.clip_factor(n, C) for n in norms])
    # (i) every clipped norm <= C
    assert np.all(c * norms <= C * (1 + 1e-15))
    assert np.any(norms < C) and np.any(norms > C)
    # (ii) C -> infinity, sigma = 0: the plain batched weight gradient (Eq. batched-grad, Format 1)
    plain, _ = O.linear_dp_grad(X, dY, 1e30, 0.0, 0)
    want = dY.reshape(B * T, D).astype(np.float64).T @ X.reshape(B * T, P).astype(np.float64)
    assert np.allclose(plain, want, rtol=1e-12, atol=1e-14)
    # (iii) below the threshold a sample contributes linearly
    k = int(np.argmin(norms))
    alpha = 0.5 * C / norms[k]            # alpha * n_k < C
    assert alpha > 1
    dY2 = dY.copy()
    dY2[k] *= np.float32(2.0)             # exact in fp32; 2 n_k still < C?
    assert 2 * norms[k] < C
    out2, norms2 = O.linear_dp_grad(X, dY2, C, 0.0, 0)
    Gk = O.per_sample_gradient(X[k], dY[k])
    assert np.allclose(out2 - out, Gk, rtol=1e-12, atol=1e-15)
    assert np.isclose(norms2[k], 2 * norms[k], rtol=1e-14)
    # (iv) above the threshold scaling a sample up changes nothing
    j = int(np.argmax(norms))
    dY3 = dY.copy()
    dY3[j] *= np.float32(4.0)
    out3, norms3 = O.linear_dp_grad(X, dY3, C, 0.0, 0)
    assert np.allclose(out3, out, rtol=1e-12, atol=1e-15) and np.isclose(norms3[j], 4 * norms[j], rtol=1e-14)
    # (v) permutations: of samples, and of tokens inside a sample
    perm = np.array([2, 0, 3, 1])
    outp, normsp = O.linear_dp_grad(X[perm], dY[perm], C, 0.0, 0)
    assert np.allclose(outp, out, rtol=1e-12, atol=1e-15) and np.allclose(normsp, norms[perm], rtol=1e-14)
    tp = np.array([5, 1, 0, 4, 2, 3])
    outt, normst = O.linear_dp_grad(X[:, tp], dY[:, tp], C, 0.0, 0)
    assert np.allclose(outt, out, rtol=1e-12, atol=1e-15) and np.allclose(normst, norms, rtol=1e-13)
    # (vi) out(sigma) - out(0) = sigma C z, the Philox field, whatever the data
    for sigma, Cn, seed, layer in ((1.0, 1.0, 1, 0), (0.8, 2.5, 99, 4)):
        o0, _ = O.linear_dp_grad(X, dY, Cn, 0.0, seed, layer)
        o1, n1 = O.linear_dp_grad(X, dY, Cn, sigma, seed, layer)
        z = O.noise_field(seed, layer, D * P).reshape(D, P)
        assert np.allclose(o1 - o0, sigma * Cn * z, rtol=1e-12, atol=1e-14)
    # noise does not touch the norms, and is added once (not per sample): B-independence of the noise part
    Xa, dYa = _rand(1, T, P, D, 8)
    oa0, _ = O.linear_dp_grad(Xa, dYa, 1.0, 0.0, 7)
    oa1, _ = O.linear_dp_grad(Xa, dYa, 1.0, 1.0, 7)
    ob0, _ = O.linear_dp_grad(X, dY, 1.0, 0.0, 7)
    ob1, _ = O.linear_dp_grad(X, dY, 1.0, 1.0, 7)
    assert np.allclose(oa1 - oa0, ob1 - ob0, rtol=0, atol=1e-14)


def test_sum_not_mean_over_batch():
    # two identical unclipped samples give twice one sample (Alg. 1: sum over b)
    X, dY = _rand(1, 3, 4, 2, 21, scale=1e-3)
    X2, dY2 = np.concatenate([X, X]), np.concatenate([dY, dY])
    o1, _ = O.linear_dp_grad(X, dY, 1.0, 0.0, 0)
    o2, _ = O.linear_dp_grad(X2, dY2, 1.0, 0.0, 0)
    assert np.allclose(o2, 2 * o1, rtol=1e-14)


def test_block_is_layerwise_independent():
    Xa, dYa = _rand(2, 4, 3, 5, 1)
    Xb, dYb = _rand(2, 4, 6, 2, 2)
    layers = [dict(X=Xa, dY=dYa, C=1.0, sigma=1.0, seed=1, layer=0),
              dict(X=Xb, dY=dYb, C=0.5, sigma=0.3, seed=2, layer=1)]
    res = O.block_dp_grad(layers)
    for L, (out, norms) in zip(layers, res):
        o, n = O.linear_dp_grad(L["X"], L["dY"], L["C"], L["sigma"], L["seed"], L["layer"])
        assert np.array_equal(o, out) and np.array_equal(n, norms)
    assert res[0][0].shape == (5, 3) and res[1][0].shape == (2, 6)


def test_workload_generator_recipe():
    w = W.WORKLOADS["gpt2_small_mlp_up"]
    small = W.scaled_down(w, B=3, T=64, dims=[(96, 160)])
    X, dY = W.make_layer(small, 0)
    assert X.dtype == np.uint16 and X.shape == (3, 64, 96) and dY.shape == (3, 64, 160)
    X2, dY2 = W.make_layer(small, 0)
    assert np.array_equal(X, X2) and np.array_equal(dY, dY2)          # seeded
    xs, dys = W.make_sample(small, 0, 1)
    assert np.array_equal(xs, X[1]) and np.array_equal(dys, dY[1])    # any sample alone
    s = W.sample_scales(small, 0)
    assert np.all((s >= 0.1) & (s <= 10))
    x64 = O.widen(X)
    assert abs(x64.std() - 1) < 0.02
    dy64 = O.widen(dY)
    for i in range(3):
        assert abs(dy64[i].std() / (math.sqrt(1e-3) * s[i]) - 1) < 0.03
    # bf16 rounding is to nearest even
    f = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e-3], np.float32)   # 1+2^-8 ties to even (1.0), 1+3*2^-8 ties up
    b = W.float32_to_bf16_bits(f)
    assert b[0] == 0x3F80 and b[1] == 0x3F80 and b[2] == 0x3F82 and b[3] == 0xBF80
    assert abs(O.widen(b[4:5])[0] - 3.0e-3) <= 2.0 ** -17   # half an ulp in [2^-9, 2^-8)


def test_accumulation_over_micro_batches_equals_the_full_batch():
    # clipping is per sample, so splitting the batch changes nothing; noise enters once
    X, dY = _rand(6, 5, 4, 3, 31)
    dY *= np.array([0.01, 30, 0.1, 3, 0.02, 8], np.float32)[:, None, None]
    full, norms = O.linear_dp_grad(X, dY, 1.0, 0.7, 5, 2)
    for split in ([2, 4], [1, 2, 3], [6], [3, 3]):
        idx = np.cumsum([0] + split)
        mbs = [(X[a:b], dY[a:b]) for a, b in zip(idx[:-1], idx[1:])]
        acc, nlist = O.accumulated_dp_grad(mbs, 1.0, 0.7, 5, 2)
        assert np.allclose(acc, full, rtol=1e-12, atol=1e-14)
        assert np.allclose(np.concatenate(nlist), norms, rtol=1e-14)
    # noise once, not once per micro-batch
    a0, _ = O.accumulated_dp_grad([(X[:3], dY[:3]), (X[3:], dY[3:])], 1.0, 0.0, 5, 2)
    a1, _ = O.accumulated_dp_grad([(X[:3], dY[:3]), (X[3:], dY[3:])], 1.0, 0.7, 5, 2)
    assert np.allclose(a1 - a0, 0.7 * O.noise_field(5, 2, 12).reshape(3, 4), rtol=1e-12, atol=1e-14)


def test_stage_by_stage_helper_of_the_gpu_tests_is_the_oracle():
    """tests/gpu_util.oracle_signal_and_bound composes the oracle's own stage functions (so that it can also return
    sum_i c_i |G_i|, the scale of the element-wise tolerance): its signal and norms must be the oracle's, bit for bit."""
    from gpu_util import oracle_signal_and_bound, elementwise_excess
    w = W.scaled_down(W.WORKLOADS["gpt2_small_mlp_up"], B=4, T=24, dims=[(40, 56)])
    X, dY = W.make_layer(w, 0)
    for C in (1.0, 1e9):
        out, norms, bound = oracle_signal_and_bound(X, dY, C)
        want, wn = O.linear_dp_grad(X, dY, C, 0.0, 1, 0)
        assert np.array_equal(out, want) and np.array_equal(norms, wn)
        assert np.all(bound >= np.abs(out) * (1 - 1e-12))
    # the tolerance itself: an error of one bfloat16 rounding per term passes, a wrong element does not
    out, norms, bound = oracle_signal_and_bound(X, dY, 1.0)
    assert elementwise_excess(out + 0.9 * 2.0 ** -8 * bound, out, bound, True)[0] <= 1.0
    bad = out.copy()
    bad[3, 5] += 3e-2 * np.sqrt(np.mean(bound ** 2)) + 2.0 ** -7 * bound[3, 5]
    worst, k = elementwise_excess(bad, out, bound, True)
    assert worst > 1.0 and divmod(k, out.shape[1]) == (3, 5)
    assert elementwise_excess(out + 2.0 ** -9 * bound, out, bound, False)[0] > 1.0
