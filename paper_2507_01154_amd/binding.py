"""ctypes binding of libflashdp.so: argument marshalling only.

Every function has the name and the arguments of the C entry point it wraps (see
include/flashdp.h).  Tensors are torch CUDA tensors used as device buffers; nothing is
computed here.  A missing library is an error: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libflashdp.so")

BF16, F32, F16 = 0, 1, 2
SCHEDULE_AUTO, SCHEDULE_TWOPASS, SCHEDULE_SCRATCH, SCHEDULE_EXPLICIT, SCHEDULE_OVERLAP, SCHEDULE_GHOST, SCHEDULE_FUSED = 0, 1, 2, 3, 4, 5, 6
_SCHEDULES = {"auto": 0, "twopass": 1, "scratch": 2, "explicit": 3, "overlap": 4, "ghost": 5, "fused": 6}

OK = 0
INVALID_ARGUMENT, MISALIGNED, UNSUPPORTED_SHAPE, WORKSPACE_TOO_SMALL, NO_DEVICE, HIP_ERROR = -1, -2, -3, -4, -5, -6


class FlashDPError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class flashdp_layer_t(ctypes.Structure):
    _fields_ = [
        ("X", ctypes.c_void_p), ("dY", ctypes.c_void_p),
        ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64),
        ("C", ctypes.c_float), ("sigma", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("layer", ctypes.c_uint32),
        ("out_grad", ctypes.c_void_p), ("out_norms", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; built by __graft_entry__.build() / build.py beforehand."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2507_01154_amd.build). "
                "There is no fallback implementation.")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, f32, u64, u32, sz, ci = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_uint64,
                                          ctypes.c_uint32, ctypes.c_size_t, ctypes.c_int)
        lp = ctypes.POINTER(flashdp_layer_t)
        L.flashdp_linear_dp_grad.argtypes = [vp, vp, i64, i64, i64, i64, f32, f32, u64, vp, vp]
        L.flashdp_linear_dp_grad.restype = ci
        L.flashdp_block_dp_grad.argtypes = [lp, ci, i64, i64, ci, ci, vp, sz, vp]
        L.flashdp_block_dp_grad.restype = ci
        L.flashdp_block_dp_grad_micro.argtypes = [lp, ci, i64, i64, ci, ci, vp, sz, vp, ci, ci]
        L.flashdp_block_dp_grad_micro.restype = ci
        L.flashdp_workspace_bytes.argtypes = [lp, ci, i64, i64, ci, ci]
        L.flashdp_workspace_bytes.restype = sz
        L.flashdp_workspace_bytes_chunked.argtypes = [lp, ci, i64, i64, ci, i64, ci]
        L.flashdp_workspace_bytes_chunked.restype = sz
        L.flashdp_last_chunk.restype = i64
        L.flashdp_linear_dp_grad_static.argtypes = [vp, vp, i64, i64, i64, i64, ci, f32, f32, u64, u32, vp, vp, vp]
        L.flashdp_linear_dp_grad_static.restype = ci
        L.flashdp_static_scratch_bytes.argtypes = []
        L.flashdp_static_scratch_bytes.restype = sz
        L.flashdp_plain_grad.argtypes = [vp, vp, i64, i64, i64, i64, ci, vp, vp]
        L.flashdp_plain_grad.restype = ci
        L.flashdp_plain_grad_balanced.argtypes = [vp, vp, i64, i64, i64, i64, ci, vp, vp, sz, vp]
        L.flashdp_plain_grad_balanced.restype = ci
        L.flashdp_plain_grad_balanced_workspace_bytes.argtypes = []
        L.flashdp_plain_grad_balanced_workspace_bytes.restype = sz
        L.flashdp_noise_field.argtypes = [u64, u32, i64, vp, vp]
        L.flashdp_noise_field.restype = ci
        L.flashdp_box_muller.argtypes = [vp, i64, vp, vp]
        L.flashdp_box_muller.restype = ci
        L.flashdp_contraction_timeline.argtypes = [vp, vp, i64, i64, i64, i64, ci, vp, sz, vp, i64, vp]
        L.flashdp_contraction_timeline.restype = i64
        L.flashdp_mfma_probe.argtypes = [ci, ci, ci, vp, vp]
        L.flashdp_mfma_probe.restype = ci
        L.flashdp_set_stream.argtypes = [vp]
        L.flashdp_set_workspace.argtypes = [vp, sz]
        L.flashdp_set_dtype.argtypes = [ci]
        L.flashdp_set_layer.argtypes = [u32]
        L.flashdp_set_schedule.argtypes = [ci]
        L.flashdp_set_stages.argtypes = [ci]
        for n in ("flashdp_set_stream", "flashdp_set_workspace", "flashdp_set_dtype", "flashdp_set_layer",
                  "flashdp_set_schedule", "flashdp_set_stages", "flashdp_release", "flashdp_version"):
            getattr(L, n).restype = ci
        L.flashdp_last_schedule.restype = ctypes.c_char_p
        L.flashdp_last_kernel.restype = ctypes.c_char_p
        L.flashdp_status_string.argtypes = [ci]
        L.flashdp_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().flashdp_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise FlashDPError(status, where)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def dtype_code(t) -> int:
    import torch
    return {torch.bfloat16: BF16, torch.float32: F32, torch.float16: F16}[t.dtype]


def schedule_code(s) -> int:
    return _SCHEDULES[s] if isinstance(s, str) else int(s)


# ---- thread-local context -------------------------------------------------------------------------

def flashdp_set_stream(stream=None):
    _check(lib().flashdp_set_stream(_stream_handle(stream)), "flashdp_set_stream")


def flashdp_set_workspace(workspace=None):
    if workspace is None:
        _check(lib().flashdp_set_workspace(None, 0), "flashdp_set_workspace")
    else:
        _check(lib().flashdp_set_workspace(_ptr(workspace), workspace.numel() * workspace.element_size()),
               "flashdp_set_workspace")


def flashdp_set_dtype(dtype: int):
    _check(lib().flashdp_set_dtype(int(dtype)), "flashdp_set_dtype")


def flashdp_set_layer(layer: int):
    _check(lib().flashdp_set_layer(int(layer)), "flashdp_set_layer")


def flashdp_set_schedule(schedule):
    _check(lib().flashdp_set_schedule(schedule_code(schedule)), "flashdp_set_schedule")


STAGE_CONTRACT, STAGE_CLIP, STAGE_AGGREGATE, STAGE_ALL = 1, 2, 4, 7


def flashdp_set_stages(mask: int = STAGE_ALL):
    _check(lib().flashdp_set_stages(int(mask)), "flashdp_set_stages")


def flashdp_release():
    _check(lib().flashdp_release(), "flashdp_release")


def flashdp_last_schedule() -> str:
    return lib().flashdp_last_schedule().decode()


def flashdp_last_kernel() -> str:
    return lib().flashdp_last_kernel().decode()


def flashdp_version() -> int:
    return lib().flashdp_version()


# ---- entry points ---------------------------------------------------------------------------------

def flashdp_linear_dp_grad(X, dY, B: int, T: int, d_in: int, d_out: int, C: float, sigma: float, seed: int,
                           out_grad, out_norms=None):
    """X [B,T,d_in], dY [B,T,d_out] device tensors of the context dtype; out_grad [d_out,d_in] fp32,
    out_norms [B] fp32 (or None).  Uses the thread's context (stream, dtype, layer, schedule, workspace)."""
    _check(lib().flashdp_linear_dp_grad(_ptr(X), _ptr(dY), B, T, d_in, d_out, C, sigma, seed,
                                        _ptr(out_grad), _ptr(out_norms)), "flashdp_linear_dp_grad")


def make_layers(layers: Sequence[dict]):
    """layers: dicts with X, dY, d_in, d_out, C, sigma, seed, layer, out_grad, out_norms (tensors or None)."""
    arr = (flashdp_layer_t * len(layers))()
    for k, L in enumerate(layers):
        arr[k].X = _ptr(L["X"])
        arr[k].dY = _ptr(L["dY"])
        arr[k].d_in = int(L["d_in"])
        arr[k].d_out = int(L["d_out"])
        arr[k].C = float(L["C"])
        arr[k].sigma = float(L["sigma"])
        arr[k].seed = int(L["seed"])
        arr[k].layer = int(L["layer"])
        arr[k].out_grad = _ptr(L["out_grad"])
        arr[k].out_norms = _ptr(L.get("out_norms"))
    return arr


def flashdp_workspace_bytes(layers, B: int, T: int, dtype: int, schedule=SCHEDULE_SCRATCH) -> int:
    arr = layers if not isinstance(layers, (list, tuple)) else make_layers(layers)
    return int(lib().flashdp_workspace_bytes(arr, len(arr), B, T, int(dtype), schedule_code(schedule)))


def flashdp_workspace_bytes_chunked(layers, B: int, T: int, dtype: int, chunk_samples: int, slots: int = 1) -> int:
    arr = layers if not isinstance(layers, (list, tuple)) else make_layers(layers)
    return int(lib().flashdp_workspace_bytes_chunked(arr, len(arr), B, T, int(dtype), int(chunk_samples), int(slots)))


def flashdp_last_chunk() -> int:
    return int(lib().flashdp_last_chunk())


def flashdp_block_dp_grad(layers, B: int, T: int, dtype: int, schedule=SCHEDULE_AUTO, workspace=None, stream=None):
    arr = layers if not isinstance(layers, (list, tuple)) else make_layers(layers)
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flashdp_block_dp_grad(arr, len(arr), B, T, int(dtype), schedule_code(schedule), ws_ptr, ws_bytes,
                                       _stream_handle(stream)), "flashdp_block_dp_grad")


def flashdp_block_dp_grad_micro(layers, B: int, T: int, dtype: int, schedule=SCHEDULE_AUTO, workspace=None, stream=None,
                                accumulate: bool = False, add_noise: bool = True):
    arr = layers if not isinstance(layers, (list, tuple)) else make_layers(layers)
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flashdp_block_dp_grad_micro(arr, len(arr), B, T, int(dtype), schedule_code(schedule), ws_ptr, ws_bytes,
                                             _stream_handle(stream), int(bool(accumulate)), int(bool(add_noise))),
           "flashdp_block_dp_grad_micro")


def flashdp_linear_dp_grad_static(X, dY, B: int, T: int, d_in: int, d_out: int, dtype: int, C: float, sigma: float,
                                  seed: int, layer: int, out_grad, out_norms=None, stream=None):
    """The entry point that allocates nothing: one layer, scratch schedule, workspace in the library's static array."""
    _check(lib().flashdp_linear_dp_grad_static(_ptr(X), _ptr(dY), B, T, d_in, d_out, int(dtype), C, sigma, seed, layer,
                                               _ptr(out_grad), _ptr(out_norms), _stream_handle(stream)),
           "flashdp_linear_dp_grad_static")


def flashdp_static_scratch_bytes() -> int:
    return int(lib().flashdp_static_scratch_bytes())


def flashdp_plain_grad(X, dY, B: int, T: int, d_in: int, d_out: int, dtype: int, out_grad, stream=None):
    _check(lib().flashdp_plain_grad(_ptr(X), _ptr(dY), B, T, d_in, d_out, int(dtype), _ptr(out_grad),
                                    _stream_handle(stream)), "flashdp_plain_grad")


def flashdp_plain_grad_balanced(X, dY, B: int, T: int, d_in: int, d_out: int, dtype: int, out_grad, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().flashdp_plain_grad_balanced(_ptr(X), _ptr(dY), B, T, d_in, d_out, int(dtype), _ptr(out_grad),
                                             _ptr(workspace), ws_bytes, _stream_handle(stream)), "flashdp_plain_grad_balanced")


def flashdp_plain_grad_balanced_workspace_bytes() -> int:
    return int(lib().flashdp_plain_grad_balanced_workspace_bytes())


def flashdp_noise_field(seed: int, layer: int, n: int, z, stream=None):
    _check(lib().flashdp_noise_field(seed, layer, n, _ptr(z), _stream_handle(stream)), "flashdp_noise_field")


def flashdp_box_muller(words, n_groups: int, z, stream=None):
    _check(lib().flashdp_box_muller(_ptr(words), n_groups, _ptr(z), _stream_handle(stream)), "flashdp_box_muller")


def flashdp_contraction_timeline(X, dY, B: int, T: int, d_in: int, d_out: int, park: bool, workspace, trace, stream=None) -> int:
    """trace: int64 device tensor of 8 words per workgroup, zeroed; returns the number of workgroups launched."""
    n = lib().flashdp_contraction_timeline(_ptr(X), _ptr(dY), B, T, d_in, d_out, int(bool(park)), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _ptr(trace), trace.numel() // 8,
                                           _stream_handle(stream))
    if n < 0:
        raise FlashDPError(int(n), "flashdp_contraction_timeline")
    return int(n)


def flashdp_mfma_probe(pattern: int, iters: int, workgroups: int, sink, stream=None):
    _check(lib().flashdp_mfma_probe(int(pattern), int(iters), int(workgroups), _ptr(sink), _stream_handle(stream)),
           "flashdp_mfma_probe")
