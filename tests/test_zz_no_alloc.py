"""The entry point that allocates nothing (flashdp_linear_dp_grad_static: scratch schedule with the workspace in
a static device array of the library) against the existing entry point (flashdp_block_dp_grad, scratch schedule,
caller-owned workspace) through the C ABI: two calls in a row on the same GPU, the second with a smaller input, so
that whatever the first call left in the shared array lies beside and behind what the second one uses.  The two
entry points share their kernels, so the outputs must be bit-identical; the first result is also held against the
CPU oracle to the tolerances of the parity suite."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import flashdp_oracle as O
import workloads as W
import paper_2507_01154_amd as F
from gpu_util import DEV, rel_fro, to_device

pytestmark = pytest.mark.gpu


def both_entry_points(B, T, P, D, sigma, seed, layer, data_seed):
    w = dataclasses.replace(W.scaled_down(W.WORKLOADS["gpt2_small_mlp_up"], B=B, T=T, dims=[(P, D)]), data_seed=data_seed)
    X, dY = W.make_layer(w, 0)
    dX, ddY = to_device(X), to_device(dY)
    res = []
    for static in (False, True):
        out = torch.full((D, P), float("nan"), device=DEV)
        norms = torch.full((B,), float("nan"), device=DEV)
        if static:
            F.flashdp_linear_dp_grad_static(dX, ddY, B, T, P, D, F.BF16, 1.0, sigma, seed, layer, out, norms)
        else:
            L = [dict(X=dX, dY=ddY, d_in=P, d_out=D, C=1.0, sigma=sigma, seed=seed, layer=layer, out_grad=out, out_norms=norms)]
            ws = torch.empty(F.flashdp_workspace_bytes(L, B, T, F.BF16, "scratch"), dtype=torch.uint8, device=DEV)
            F.flashdp_block_dp_grad(L, B, T, F.BF16, "scratch", ws)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), norms.cpu().numpy()))
    return X, dY, res


def test_static_entry_point_matches_the_allocating_one_on_two_calls_in_a_row():
    assert F.flashdp_static_scratch_bytes() == 64 << 20
    # first call: several 256x256 tiles with ragged edges, the large-shape kernel (B * tiles >= 128 work items)
    X, dY, (ref, got) = both_entry_points(B=6, T=200, P=1160, D=1320, sigma=1.0, seed=9, layer=4, data_seed=21)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    sig, wn = O.linear_dp_grad(X, dY, 1.0, 0.0, 9, 4)
    z = O.noise_field(9, 4, sig.size).reshape(sig.shape)
    assert rel_fro(got[0] - z, sig) <= 4e-3
    assert np.max(np.abs(got[1] - wn) / wn) <= 1e-4
    # second call, smaller in every dimension (the small-shape kernel): reads nothing of what the first one left
    X, dY, (ref, got) = both_entry_points(B=3, T=70, P=328, D=264, sigma=0.5, seed=2, layer=1, data_seed=22)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    sig, wn = O.linear_dp_grad(X, dY, 1.0, 0.0, 2, 1)
    z = O.noise_field(2, 1, sig.size).reshape(sig.shape)
    assert rel_fro(got[0] - 0.5 * z, sig) <= 4e-3
    assert np.max(np.abs(got[1] - wn) / wn) <= 1e-4


def test_static_entry_point_rejects_what_does_not_fit():
    # the Llama-7B q_proj layer at B = 4 needs 128 MiB of parked tiles: refused before anything is enqueued
    t = torch.zeros(16, dtype=torch.bfloat16, device=DEV)
    o = torch.zeros(4, device=DEV)
    with pytest.raises(F.FlashDPError) as ei:
        F.flashdp_linear_dp_grad_static(t, t, 4, 2048, 4096, 4096, F.BF16, 1.0, 1.0, 1, 0, o, None)
    assert ei.value.status == F.WORKSPACE_TOO_SMALL
    # exactly at the limit of what fits: B * S * 2 bytes of tiles plus the small header
    L = [dict(X=None, dY=None, d_in=768, d_out=3072, C=1.0, sigma=1.0, seed=0, layer=0, out_grad=None)]
    assert F.flashdp_workspace_bytes(L, 8, 1024, F.BF16, "scratch") <= F.flashdp_static_scratch_bytes()
