"""The autograd wrapper: a two-layer MLP trained with a per-sample-summed loss gets, on each weight, the
oracle's clipped and noised gradient computed from the activations and output gradients of the same step."""
import numpy as np
import pytest
import torch

from oracle import flashdp_oracle as O
from gpu_util import DEV, rel_fro

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def test_two_layer_mlp_backward_matches_oracle():
    from paper_2507_01154_amd.autograd import DPLinear
    torch.manual_seed(0)
    B, T, d0, d1, d2 = 4, 48, 72, 136, 40
    l1 = DPLinear(d0, d1, C=0.05, sigma=0.5, seed=3, layer=0, device=DEV)
    l2 = DPLinear(d1, d2, C=0.05, sigma=0.5, seed=3, layer=1, device=DEV)
    l1.step = l2.step = 7
    x = torch.randn(B, T, d0, device=DEV).bfloat16()
    target = torch.randn(B, T, d2, device=DEV).bfloat16()
    # the same network in plain torch, to capture X and dY of each layer
    w1 = l1.weight.detach().clone().requires_grad_(True)
    w2 = l2.weight.detach().clone().requires_grad_(True)
    a1 = (x @ w1.t())
    a1.retain_grad()
    y2 = torch.relu(a1) @ w2.t()
    y2.retain_grad()
    (((y2.float() - target.float()) ** 2).sum()).backward()
    # the DP network
    h = torch.relu(l1(x))
    y = l2(h)
    (((y.float() - target.float()) ** 2).sum()).backward()
    torch.cuda.synchronize()
    cases = [(l1, x, a1.grad, d0, d1), (l2, torch.relu(a1).detach(), y2.grad, d1, d2)]
    for lin, X, dY, di, do in cases:
        sig, wn = O.linear_dp_grad(_bits(X), _bits(dY), lin.C, 0.0, lin.noise_seed(), lin.layer)
        z = O.noise_field(lin.noise_seed(), lin.layer, do * di).reshape(do, di)
        want = sig + lin.sigma * lin.C * z
        got = lin.weight.grad.float().cpu().numpy()
        # weight.grad is rounded to the parameter dtype (bf16): 2^-9 relative per element
        assert rel_fro(got, want) <= 1e-2
        assert np.max(np.abs(lin.last_norms.cpu().numpy() - wn) / wn) <= 1e-4
        assert np.any(wn > lin.C) and got.shape == (do, di)
    # the seed folds the step in: another step, another noise
    assert l1.noise_seed() != DPLinear(d0, d1, seed=3, device=DEV).noise_seed()


def test_deferred_block_call_gives_the_same_gradients():
    """Inside deferred_weight_grads the layers of one backward pass go to the library in a single per-block call
    (overlapped schedule when the shapes allow); the gradients are the ones the layer-by-layer calls produce."""
    from paper_2507_01154_amd.autograd import DPLinear, deferred_weight_grads
    import paper_2507_01154_amd as F
    torch.manual_seed(1)
    B, T, d0, d1, d2 = 4, 64, 1024, 1536, 1024
    l1 = DPLinear(d0, d1, C=0.05, sigma=0.5, seed=5, layer=0, device=DEV)
    l2 = DPLinear(d1, d2, C=0.05, sigma=0.5, seed=5, layer=1, device=DEV)
    x = torch.randn(B, T, d0, device=DEV).bfloat16()
    target = torch.randn(B, T, d2, device=DEV).bfloat16()

    def run():
        l1.weight.grad = l2.weight.grad = None
        y = l2(torch.relu(l1(x)))
        (((y.float() - target.float()) ** 2).sum()).backward()

    run()
    torch.cuda.synchronize()
    ref = [l1.weight.grad.clone(), l2.weight.grad.clone()]
    ref_norms = [l1.last_norms.clone(), l2.last_norms.clone()]
    with deferred_weight_grads():
        run()
        assert l1.weight.grad is None and l2.weight.grad is None      # nothing computed yet
    torch.cuda.synchronize()
    assert F.flashdp_last_schedule() in ("overlap", "scratch")
    assert torch.equal(l1.weight.grad, ref[0]) and torch.equal(l2.weight.grad, ref[1])
    assert torch.equal(l1.last_norms, ref_norms[0]) and torch.equal(l2.last_norms, ref_norms[1])
    # a second deferred pass without clearing adds to .grad, as autograd would
    with deferred_weight_grads():
        y = l2(torch.relu(l1(x)))
        (((y.float() - target.float()) ** 2).sum()).backward()
    torch.cuda.synchronize()
    assert torch.allclose(l1.weight.grad.float(), 2 * ref[0].float(), rtol=2e-2, atol=1e-3)
