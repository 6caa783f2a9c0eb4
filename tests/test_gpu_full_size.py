"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (one flashdp_block_dp_grad call over all layers of the workload, caller-owned workspace, schedule
auto).  The signal (sigma = 0) and the norms are compared with the full fp64 oracle element by element;
the noise is compared on sampled elements the oracle computes one by one (2^20 random indices plus the
first and last 4096 of each layer)."""
import numpy as np
import pytest
import torch

from oracle import flashdp_oracle as O
import workloads as W
import paper_2507_01154_amd as F
from gpu_util import DEV, rel_fro, to_device, oracle_signal_and_bound, elementwise_excess

pytestmark = pytest.mark.gpu


def run_workload(w, sigma, schedule="auto"):
    layers, host = [], []
    for l, spec in enumerate(w.layers):
        X, dY = W.make_layer(w, l)
        out = torch.full((spec.d_out, spec.d_in), float("nan"), device=DEV)
        norms = torch.full((w.B,), float("nan"), device=DEV)
        layers.append(dict(X=to_device(X), dY=to_device(dY), d_in=spec.d_in, d_out=spec.d_out, C=w.C, sigma=sigma,
                           seed=w.layer_seed(l), layer=l, out_grad=out, out_norms=norms))
        host.append((X, dY))
    arr = F.make_layers(layers)
    dt = {"bf16": F.BF16, "f16": F.F16, "fp32": F.F32}[w.dtype]
    ws = torch.empty(F.flashdp_workspace_bytes(arr, w.B, w.T, dt, "scratch"), dtype=torch.uint8, device=DEV)
    F.flashdp_block_dp_grad(arr, w.B, w.T, dt, schedule, ws)
    torch.cuda.synchronize()
    used = F.flashdp_last_schedule()
    outs = [(L["out_grad"].cpu().numpy(), L["out_norms"].cpu().numpy()) for L in layers]
    return host, outs, used


def check_layer(w, l, X, dY, got0, gn, got1, used):
    spec = w.layers[l]
    S = spec.d_in * spec.d_out
    if X.dtype == np.float16:      # the oracle takes the stored values widened exactly
        X, dY = X.astype(np.float32), dY.astype(np.float32)
    sig, wn, bound = oracle_signal_and_bound(X, dY, w.C)     # bit-identical to O.linear_dp_grad(..., sigma = 0) (CPU suite)
    e_sig = rel_fro(got0, sig)
    parked = w.dtype != "fp32" and used in ("scratch", "overlap", "fused")     # bfloat16 scratch for both 16-bit input types
    worst, k = elementwise_excess(got0, sig, bound, parked)
    assert worst <= 1.0, (f"{spec.name} element {divmod(k, spec.d_in)}: got {got0.reshape(-1)[k]!r}, want {sig.reshape(-1)[k]!r}, "
                          f"sum_i c_i|G_i| {bound.reshape(-1)[k]!r}, error / allowed = {worst:.3f}")
    del bound
    e_norm = float(np.max(np.abs(gn - wn) / wn))
    tol = 1e-4 if w.dtype == "fp32" else 1e-2
    tight = 4e-3 if (w.dtype != "fp32" and used in ("scratch", "fused")) else 5e-5
    assert e_sig <= tol and e_sig <= tight, (spec.name, e_sig)
    assert e_norm <= 5e-3 and e_norm <= 1e-4, (spec.name, e_norm)
    rng = np.random.default_rng(100 + l)
    idx = np.unique(np.concatenate([np.arange(min(4096, S)), np.arange(max(0, S - 4096), S),
                                    rng.integers(0, S, size=1 << 20)]))
    z = O.noise_at(w.layer_seed(l), l, idx)
    scale = w.sigma * w.C
    d = got1.reshape(-1)[idx].astype(np.float64) - got0.reshape(-1)[idx].astype(np.float64)
    assert np.max(np.abs(d - scale * z)) <= 4e-6 * scale, spec.name
    want1 = sig.reshape(-1)[idx] + scale * z
    assert np.linalg.norm(got1.reshape(-1)[idx] - want1) / np.linalg.norm(want1) <= tol, spec.name
    # every sample clips in these workloads: the clipped batch sum cannot be longer than B * C
    assert np.all(gn > w.C) and np.linalg.norm(got0.astype(np.float64)) <= w.B * w.C * (1 + 1e-6)
    print(f"{w.name}/{spec.name}: schedule {used}, signal rel err {e_sig:.2e}, norm rel err {e_norm:.2e}, norms {wn.min():.3g}..{wn.max():.3g}")


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name", ["gpt2_small_mlp_up", "llama7b_q_proj", "llama13b_up_proj"])
def test_single_layer_configs_full_size(name):
    w = W.WORKLOADS[name]
    host, o0, used = run_workload(w, 0.0)
    _, o1, _ = run_workload(w, w.sigma)
    assert used == "scratch"
    X, dY = host[0]
    check_layer(w, 0, X, dY, o0[0][0], o0[0][1], o1[0][0], used)
    assert np.array_equal(o0[0][1], o1[0][1])


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name", ["llama7b_q_proj_fp32", "llama7b_q_proj_f16"])
def test_precision_variants_full_size_llama7b(name):
    """The mixed-precision experiment's other input types (Appendix D.2) at the full Llama-7B q_proj size: fp32 inputs
    through the fp32 matrix-core kernel with an fp32 scratch (stated tolerance 1e-4, derived 5e-5), fp16 inputs
    through the 16-bit kernel with the bfloat16 scratch."""
    w = W.WORKLOADS[name]
    host, o0, used = run_workload(w, 0.0)
    _, o1, _ = run_workload(w, w.sigma)
    assert used == "scratch"
    X, dY = host[0]
    check_layer(w, 0, X, dY, o0[0][0], o0[0][1], o1[0][0], used)
    assert np.array_equal(o0[0][1], o1[0][1])


@pytest.fixture(scope="module")
def block_runs():
    w = W.WORKLOADS["llama13b_block"]
    host, o0, used = run_workload(w, 0.0)
    _, o1, _ = run_workload(w, w.sigma)
    return w, host, o0, o1, used


@pytest.mark.timeout(600)
@pytest.mark.parametrize("l", range(7))
def test_llama13b_block_full_size(block_runs, l):
    w, host, o0, o1, used = block_runs
    assert used == "scratch"
    X, dY = host[l]
    check_layer(w, l, X, dY, o0[l][0], o0[l][1], o1[l][0], used)


@pytest.mark.timeout(300)
def test_two_pass_schedule_full_size_llama7b():
    w = W.WORKLOADS["llama7b_q_proj"]
    host, o0, used = run_workload(w, 0.0, "twopass")
    _, o1, _ = run_workload(w, w.sigma, "twopass")
    assert used == "twopass"
    X, dY = host[0]
    check_layer(w, 0, X, dY, o0[0][0], o0[0][1], o1[0][0], used)


@pytest.mark.timeout(300)
def test_explicit_four_stage_schedule_full_size_llama7b():
    w = W.WORKLOADS["llama7b_q_proj"]
    host, o0, used = run_workload_sched(w, 0.0, "explicit")
    _, o1, _ = run_workload_sched(w, w.sigma, "explicit")
    assert used == "explicit"
    X, dY = host[0]
    check_layer(w, 0, X, dY, o0[0][0], o0[0][1], o1[0][0], used)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name", ["gpt2_small_mlp_up", "llama7b_q_proj"])
def test_ghost_norm_schedule_full_size(name):
    w = W.WORKLOADS[name]
    host, o0, used = run_workload_sched(w, 0.0, "ghost")
    _, o1, _ = run_workload_sched(w, w.sigma, "ghost")
    assert used == "ghost"
    X, dY = host[0]
    check_layer(w, 0, X, dY, o0[0][0], o0[0][1], o1[0][0], used)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("name", ["gpt2_small_mlp_up", "llama7b_q_proj"])
def test_fused_single_launch_schedule_full_size(name):
    """Algorithm 1 in one launch with a grid barrier, at the sizes where every tile has a workgroup on the chip:
    36 tiles (GPT-2) and 256 tiles (Llama-7B q_proj: every compute unit holds one)."""
    w = W.WORKLOADS[name]
    host, o0, used = run_workload_sched(w, 0.0, "fused")
    assert used == "fused" and F.flashdp_last_kernel() == "fused_dp_kernel"
    _, o1, _ = run_workload_sched(w, w.sigma, "fused")
    X, dY = host[0]
    check_layer(w, 0, X, dY, o0[0][0], o0[0][1], o1[0][0], used)
    assert np.array_equal(o0[0][1], o1[0][1])


def run_workload_sched(w, sigma, schedule):
    """run_workload with a workspace sized for the given schedule."""
    layers, host = [], []
    for l, spec in enumerate(w.layers):
        X, dY = W.make_layer(w, l)
        out = torch.full((spec.d_out, spec.d_in), float("nan"), device=DEV)
        norms = torch.full((w.B,), float("nan"), device=DEV)
        layers.append(dict(X=to_device(X), dY=to_device(dY), d_in=spec.d_in, d_out=spec.d_out, C=w.C, sigma=sigma,
                           seed=w.layer_seed(l), layer=l, out_grad=out, out_norms=norms))
        host.append((X, dY))
    arr = F.make_layers(layers)
    ws = torch.empty(F.flashdp_workspace_bytes(arr, w.B, w.T, F.BF16, schedule), dtype=torch.uint8, device=DEV)
    F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, schedule, ws)
    torch.cuda.synchronize()
    outs = [(L["out_grad"].cpu().numpy(), L["out_norms"].cpu().numpy()) for L in layers]
    return host, outs, F.flashdp_last_schedule()


@pytest.mark.timeout(600)
def test_overlapped_schedule_is_bit_identical_to_scratch(block_runs):
    """The overlapped schedule reorders kernels across two streams, nothing else: same bits as the scratch
    schedule, on repeated calls (events and scratch slots are reused), and noise included."""
    w, host, o0, o1, used = block_runs
    layers = []
    for l, spec in enumerate(w.layers):
        X, dY = host[l]
        out = torch.full((spec.d_out, spec.d_in), float("nan"), device=DEV)
        norms = torch.full((w.B,), float("nan"), device=DEV)
        layers.append(dict(X=to_device(X), dY=to_device(dY), d_in=spec.d_in, d_out=spec.d_out, C=w.C, sigma=w.sigma,
                           seed=w.layer_seed(l), layer=l, out_grad=out, out_norms=norms))
    arr = F.make_layers(layers)
    need = F.flashdp_workspace_bytes(arr, w.B, w.T, F.BF16, "overlap")
    assert need >= 2 * F.flashdp_workspace_bytes(arr, w.B, w.T, F.BF16, "scratch") - 512
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    for rep in range(3):
        for L in layers:
            L["out_grad"].fill_(float("nan"))
        F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, "auto" if rep == 2 else "overlap", ws)
        torch.cuda.synchronize()
        assert F.flashdp_last_schedule() == "overlap"
        for l, L in enumerate(layers):
            assert np.array_equal(L["out_grad"].cpu().numpy(), o1[l][0]), (rep, l)
            assert np.array_equal(L["out_norms"].cpu().numpy(), o1[l][1]), (rep, l)
    # a workspace with one slot only: auto stays on the scratch schedule; an explicit request is refused
    F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, "auto", ws[: need // 2])
    torch.cuda.synchronize()
    assert F.flashdp_last_schedule() == "scratch"
    with pytest.raises(F.FlashDPError) as ei:
        F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, "overlap", ws[: need // 2])
    assert ei.value.status == F.WORKSPACE_TOO_SMALL
    # a single layer has nothing to overlap with
    one = F.make_layers(layers[:1])
    F.flashdp_block_dp_grad(one, w.B, w.T, F.BF16, "overlap", ws)
    torch.cuda.synchronize()
    assert F.flashdp_last_schedule() == "scratch"
    assert np.array_equal(layers[0]["out_grad"].cpu().numpy(), o1[0][0])


@pytest.mark.timeout(600)
def test_bounded_memory_scratch_full_size_llama13b_up_proj():
    """A workspace that holds two parked samples of the Llama-13B up_proj layer (as much memory as out_grad itself)
    instead of the whole batch of eight: AUTO goes through the batch in chunks of two samples instead of computing every
    G_i twice; with room for four, in two overlapped slots of two.  Oracle parity as for the full scratch, and the
    time beside the full-scratch time (printed; asserted loosely, the measured figure is in the design notes)."""
    import dataclasses
    w = dataclasses.replace(W.WORKLOADS["llama13b_up_proj"], B=8)
    spec = w.layers[0]
    X, dY = W.make_layer(w, 0)
    dX, ddY = to_device(X), to_device(dY)
    out = torch.full((spec.d_out, spec.d_in), float("nan"), device=DEV)
    norms = torch.full((w.B,), float("nan"), device=DEV)
    L = dict(X=dX, dY=ddY, d_in=spec.d_in, d_out=spec.d_out, C=w.C, sigma=0.0, seed=w.layer_seed(0), layer=0, out_grad=out, out_norms=norms)
    full = F.flashdp_workspace_bytes([L], w.B, w.T, F.BF16, "scratch")
    sig = wn = bound = None

    def timed(arr, ws, reps=5):
        F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, "auto", ws)
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(reps):
            F.flashdp_block_dp_grad(arr, w.B, w.T, F.BF16, "auto", ws)
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / reps

    arr = F.make_layers([L])
    ws_full = torch.empty(full, dtype=torch.uint8, device=DEV)
    t_full = timed(arr, ws_full)
    assert F.flashdp_last_schedule() == "scratch" and F.flashdp_last_chunk() == w.B
    ref = out.cpu().numpy()
    ref_n = norms.cpu().numpy()
    del ws_full
    for chunk, slots, want in ((2, 1, "scratch"), (2, 2, "overlap")):
        need = F.flashdp_workspace_bytes_chunked([L], w.B, w.T, F.BF16, chunk, slots)
        assert need <= slots * (4 * spec.d_in * spec.d_out + (1 << 20)) and need <= slots * full // 3   # one slot: as much memory as out_grad, a quarter of the full scratch
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        out.fill_(float("nan"))
        t = timed(arr, ws)
        assert F.flashdp_last_schedule() == want and F.flashdp_last_chunk() == chunk
        got, gn = out.cpu().numpy(), norms.cpu().numpy()
        assert np.array_equal(gn, ref_n)                              # same kernels on the same samples
        assert rel_fro(got, ref.astype(np.float64)) <= 1e-6           # the same sum in another fp32 order
        if sig is None:
            sig, wn, bound = oracle_signal_and_bound(X, dY, w.C)
        assert rel_fro(got, sig) <= 4e-3 and np.max(np.abs(gn - wn) / wn) <= 1e-4
        worst, k = elementwise_excess(got, sig, bound, True)
        assert worst <= 1.0, (divmod(k, spec.d_in), worst)
        print(f"up_proj B=8, workspace {need / 2**20:.0f} MiB ({chunk} sample(s) x {slots} slot(s), {want}): {t:.3f} ms vs full scratch ({full / 2**20:.0f} MiB) {t_full:.3f} ms = {t / t_full:.3f}x")
        assert t <= 1.25 * t_full
        del ws
