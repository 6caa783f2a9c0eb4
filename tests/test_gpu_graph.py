"""The library only enqueues kernels (and, for the overlapped schedule, event records/waits between its two
streams), so a call can be captured into a HIP graph when the caller supplies the workspace.  Replays are
checked against the eager result, several times, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import workloads as W
import paper_2507_01154_amd as F
from gpu_util import DEV, to_device

pytestmark = pytest.mark.gpu


def _layers(w, dims_idx):
    layers = []
    for l in dims_idx:
        spec = w.layers[l]
        X, dY = W.make_layer(w, l)
        layers.append(dict(X=to_device(X), dY=to_device(dY), d_in=spec.d_in, d_out=spec.d_out, C=w.C, sigma=w.sigma,
                           seed=w.layer_seed(l), layer=l,
                           out_grad=torch.zeros((spec.d_out, spec.d_in), device=DEV),
                           out_norms=torch.zeros((w.B,), device=DEV)))
    return layers


@pytest.mark.parametrize("schedule,case", [("scratch", "gpt2"), ("twopass", "gpt2"), ("overlap", "block2"), ("fused", "gpt2")])
def test_graph_capture_and_replay(schedule, case):
    if case == "gpt2":
        w = W.WORKLOADS["gpt2_small_mlp_up"]
        layers = _layers(w, [0])
    else:
        base = W.WORKLOADS["llama13b_block"]
        # large enough for the 256x256 path (many 256 x 256 work items per layer), which the overlapped schedule needs
        w = W.scaled_down(base, B=8, T=128, dims=[(2048, 4096), (4096, 2048), (2048, 4096)])
        layers = _layers(w, [0, 1, 2])
    arr = F.make_layers(layers)
    ws = torch.empty(F.flashdp_workspace_bytes(arr, w.B, w.T, F.BF16, schedule), dtype=torch.uint8, device=DEV)
    # eager reference (also sets the kernels' launch attributes outside the capture)
    F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, schedule, ws)
    torch.cuda.synchronize()
    used = F.flashdp_last_schedule()
    assert used == schedule
    want = [(L["out_grad"].clone(), L["out_norms"].clone()) for L in layers]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, schedule, ws)
    assert F.flashdp_last_schedule() == used
    for rep in range(4):
        for L in layers:
            L["out_grad"].fill_(float("nan"))
            L["out_norms"].fill_(float("nan"))
        ws.random_(0, 255)                      # eager work between replays: the graph must not depend on old scratch
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for L, (og, on) in zip(layers, want):
            assert torch.equal(L["out_grad"], og), (schedule, rep)
            assert torch.equal(L["out_norms"], on), (schedule, rep)
