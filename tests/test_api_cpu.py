"""CPU-side checks of the boundary: the shared library loads, exports every symbol the header
declares, and rejects bad arguments before touching a device.  No kernel is launched here."""
import ctypes
import os
import re

import pytest
import torch

import paper_2507_01154_amd as F

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "flashdp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(flashdp_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert "flashdp_linear_dp_grad" in names and "flashdp_block_dp_grad" in names and len(names) >= 14
    L = F.lib()
    for n in names:
        assert hasattr(L, n), n
    assert F.flashdp_version() >= 100
    assert F.status_string(0) == "ok" and "workspace" in F.status_string(F.WORKSPACE_TOO_SMALL)


def test_binding_wraps_every_entry_point_by_name():
    for n in declared_functions():
        if n in ("flashdp_status_string",):
            continue
        assert hasattr(F, n), n


A, B_, O_ = 0x10000, 0x20000, 0x30000      # fake, aligned, never dereferenced: every call below fails validation first


@pytest.mark.parametrize("args,want", [
    ((None, B_, 1, 1, 8, 8, 1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, None, 1, 1, 8, 8, 1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, 1.0, 0.0, 0, None, None), F.INVALID_ARGUMENT),
    ((A, B_, 0, 1, 8, 8, 1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, -3, 8, 8, 1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 0, 8, 1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 0, 1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, 0.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, -1.0, 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, float("nan"), 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, float("inf"), 0.0, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, 1.0, -0.5, 0, O_, None), F.INVALID_ARGUMENT),
    ((A, B_, 1, 1, 8, 8, 1.0, float("nan"), 0, O_, None), F.INVALID_ARGUMENT),
    ((A + 8, B_, 1, 1, 8, 8, 1.0, 0.0, 0, O_, None), F.MISALIGNED),
    ((A, B_ + 2, 1, 1, 8, 8, 1.0, 0.0, 0, O_, None), F.MISALIGNED),
    ((A, B_, 1, 1, 8, 8, 1.0, 0.0, 0, O_ + 4, None), F.MISALIGNED),
    ((A, B_, 1, 1 << 20, 1 << 12, 8, 1.0, 0.0, 0, O_, None), F.UNSUPPORTED_SHAPE),
    ((A, B_, 1, 4, 8, 1 << 31, 1.0, 0.0, 0, O_, None), F.UNSUPPORTED_SHAPE),
])
def test_argument_validation(args, want):
    assert F.lib().flashdp_linear_dp_grad(*args) == want


def test_context_setters_validate():
    L = F.lib()
    assert L.flashdp_set_dtype(7) == F.INVALID_ARGUMENT and L.flashdp_set_dtype(F.BF16) == F.OK
    assert L.flashdp_set_schedule(9) == F.INVALID_ARGUMENT and L.flashdp_set_schedule(0) == F.OK
    assert L.flashdp_set_workspace(None, 16) == F.INVALID_ARGUMENT
    assert L.flashdp_set_workspace(0x1008, 64) == F.MISALIGNED
    assert L.flashdp_set_workspace(None, 0) == F.OK
    assert L.flashdp_block_dp_grad(None, 1, 1, 1, 0, 0, None, 0, None) == F.INVALID_ARGUMENT
    assert L.flashdp_plain_grad(A, B_, 1, 1, 8, 8, 5, O_, None) == F.INVALID_ARGUMENT
    assert L.flashdp_noise_field(1, 0, 0, O_, None) == F.INVALID_ARGUMENT
    assert L.flashdp_box_muller(None, 4, O_, None) == F.INVALID_ARGUMENT


def test_workspace_bytes_formula():
    mk = lambda p, d: dict(X=None, dY=None, d_in=p, d_out=d, C=1.0, sigma=1.0, seed=0, layer=0, out_grad=None)
    B, T = 8, 2048
    big = F.flashdp_workspace_bytes([mk(5120, 13824), mk(5120, 5120)], B, T, F.BF16, "scratch")
    assert big >= B * 5120 * 13824 * 2 and big < B * 5120 * 13824 * 2 + (1 << 20)      # 16-bit scratch of the largest layer
    assert F.flashdp_workspace_bytes([mk(5120, 13824)], B, T, F.F32, "scratch") >= B * 5120 * 13824 * 4
    assert 0 < F.flashdp_workspace_bytes([mk(5120, 13824)], B, T, F.BF16, "twopass") < (1 << 20)
    assert F.flashdp_workspace_bytes([mk(0, 8)], B, T, F.BF16, "scratch") == 0
    # ghost-norm schedule: one partial per 128-row block pair on or above the diagonal (T = 2048: 136 per sample)
    ghost = F.flashdp_workspace_bytes([mk(5120, 5120)], B, T, F.BF16, "ghost")
    nb = (T + 127) // 128
    assert B * max(nb * (nb + 1) // 2, 400) * 4 <= ghost < (1 << 20)
    L = F.lib()
    assert L.flashdp_set_schedule(6) == F.OK and L.flashdp_set_schedule(7) == F.INVALID_ARGUMENT
    assert L.flashdp_set_schedule(0) == F.OK


def test_tile_shape_follows_the_rounds_of_equally_long_work_items(monkeypatch):
    # host logic only, read off the number of norm partials (B x tiles floats, rounded up to 256 bytes) in the two-pass
    # workspace.  Without a device 256 compute units are assumed.
    mk = lambda p, d: [dict(X=None, dY=None, d_in=p, d_out=d, C=1.0, sigma=1.0, seed=0, layer=0, out_grad=None)]

    def partial_bytes(p, d, B, T, tile=None):
        if tile is None:
            monkeypatch.delenv("FLASHDP_TILE", raising=False)
        else:
            monkeypatch.setenv("FLASHDP_TILE", str(tile))
        n = F.flashdp_workspace_bytes(mk(p, d), B, T, F.BF16, "twopass")
        monkeypatch.delenv("FLASHDP_TILE", raising=False)
        return n - 256          # the clip factors take the first 256 bytes (B <= 64)

    up = lambda n: (n + 255) // 256 * 256
    # 768 -> 3072 at B = 8: 36 tiles of 256 x 256 (288 items, two rounds) against 32 of 384 x 192 (256 items, one round)
    assert partial_bytes(768, 3072, 8, 1024, tile=6) == up(8 * 36 * 4)
    assert partial_bytes(768, 3072, 8, 1024) == up(8 * 32 * 4)
    assert partial_bytes(3072, 768, 8, 1024) == up(8 * 32 * 4)              # transposed: 192 x 384
    assert partial_bytes(768, 3072, 8, 1024, tile=7) == up(8 * 32 * 4)
    # the Llama shapes keep 256 x 256: 400 / 1080 / 256 tiles
    assert partial_bytes(5120, 5120, 8, 2048) == up(8 * 400 * 4)
    assert partial_bytes(5120, 13824, 8, 2048) == up(8 * 1080 * 4)
    assert partial_bytes(4096, 4096, 4, 2048) == up(4 * 256 * 4)
    # equal tile-rounds (1024 x 3072 at B = 8: 384 items either way): the square tile stays
    assert partial_bytes(1024, 3072, 8, 1024) == up(8 * 48 * 4)


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful on a host without a GPU")
def test_no_device_is_an_error_not_a_crash():
    assert F.lib().flashdp_linear_dp_grad(A, B_, 1, 1, 8, 8, 1.0, 0.0, 0, O_, None) == F.NO_DEVICE
    assert F.lib().flashdp_noise_field(1, 0, 16, O_, None) == F.NO_DEVICE


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_header_is_plain_c_and_links(tmp_path):
    import subprocess
    exe = str(tmp_path / "abi_check")
    lib_dir = os.path.join(ROOT, "paper_2507_01154_amd")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-o", exe, os.path.join(ROOT, "tests", "abi_check.c"),
                           "-L" + lib_dir, "-lflashdp", "-Wl,-rpath," + lib_dir])
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.split()[0] == str(F.flashdp_version())


def test_register_budget_of_the_overlapped_schedule():
    """The overlapped schedule runs two 4-wave aggregation workgroups per CU beside one resident 8-wave
    contraction workgroup.  That only fits while, per SIMD, 2 contraction waves + 2 aggregation waves stay within
    the 512 vector registers (allocated in blocks of 8); a contraction kernel grown to 218 registers measured
    4 % slower end to end for this reason alone.  Checked from the compiler's own resource report."""
    import re
    import subprocess
    import tempfile
    from paper_2507_01154_amd import build as B
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "--cuda-device-only", "-c",
               "-Rpass-analysis=kernel-resource-usage", B.sources()[0], "-o", os.path.join(tmp, "api.o")]
        res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    usage, cur = {}, None
    for line in res.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = m.group(1)
            usage[cur] = {}
        m = re.search(r"remark:\s+(VGPRs|AGPRs|VGPRs Spill|SGPRs Spill|ScratchSize \[bytes/lane\]): (\d+)", line)
        if m and cur:
            usage[cur][m.group(1)] = int(m.group(2))
    up8 = lambda n: (n + 7) // 8 * 8
    # MODE_SPILL, bf16 and f16, untraced, of the two 256 x 256 direct-to-LDS kernels (16x16x32: the default; 32x32x16)
    spill = [k for k in usage if ("gemm_mfma_dma_kernel" in k or "gemm_mfma_dma16_kernel" in k) and "ELi1ELi" in k and k.endswith("Lb0EEEvNS_8GemmArgsE")]
    # the streaming kernels that run beside it: the bounded-grid forms (clip factors folded in, one load in flight; and
    # the plain one used when the factors come from a launch of their own)
    agg = [k for k in usage if "aggregate16_persistent_kernel" in k or ("clip_aggregate16_kernel" in k and "Lb0EEE" in k)]
    assert len(spill) == 4 and len(agg) == 2
    # one aggregation workgroup per CU = one of its waves per SIMD beside two contraction waves
    for k in spill:
        for g in agg:
            assert 2 * up8(usage[k]["VGPRs"] + usage[k]["AGPRs"]) + up8(usage[g]["VGPRs"]) <= 512, (k, usage[k], g, usage[g])
    # and no kernel of the library spills registers to memory - except the single-launch comparison kernel, which keeps
    # a dozen values of its sample-boundary code in memory across the main loop (none is touched inside the loop)
    for k, u in usage.items():
        if "fused_dp_kernel" in k:
            assert u.get("ScratchSize [bytes/lane]", 0) <= 64, (k, u)
            continue
        assert u.get("VGPRs Spill", 0) == 0 and u.get("ScratchSize [bytes/lane]", 0) == 0, (k, u)
