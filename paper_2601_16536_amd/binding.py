"""ctypes binding of libw4a16.so: the names of include/w4a16.h, argument
marshalling only.  torch supplies device memory and the stream handle; every
step of the computation runs inside the HIP library.  There is no fallback: if
the library is not built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libw4a16.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_GROUP, ERR_ALIGN, ERR_WORKSPACE, ERR_HIP, ERR_UNSUPPORTED = range(1, 8)
KERNEL_AUTO, KERNEL_WAVE_SPLIT, KERNEL_STRIPE, KERNEL_TILE = -1, 0, 3, 4  # 1 and 2: retired families

EXPORTS = (
    "w4a16_gemm", "w4a16_gemm_ex", "w4a16_gemm_ws", "w4a16_gemm_noalloc", "w4a16_gemm_bf16", "w4a16_set_workspace", "w4a16_tune",
    "w4a16_workspace_bytes", "w4a16_query_plan",
    "w4a16_reduce", "w4a16_dequant", "w4a16_quantize", "w4a16_stream_probe", "w4a16_status_string", "w4a16_last_hip_error", "w4a16_shutdown",
)


class Plan(ctypes.Structure):
    _fields_ = [
        ("kernel", ctypes.c_int), ("split", ctypes.c_int), ("groups_per_split", ctypes.c_int),
        ("tile_n", ctypes.c_int), ("tile_m", ctypes.c_int), ("waves_k", ctypes.c_int), ("workgroups", ctypes.c_int),
        ("threads", ctypes.c_int), ("workspace_bytes", ctypes.c_size_t),
    ]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class W4A16Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = "%s: %s" % (where, status_string(status))
        hip = last_hip_error()
        if hip:
            msg += " (%s)" % hip
        super().__init__(msg)


_lib = None


def use_library(path: str) -> None:
    """Loads another build of the library (the profiling build libw4a16_timeline.so) instead of libw4a16.so.
    Only before the first call into the library."""
    global LIB_PATH
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    LIB_PATH = path


def lib():
    """The loaded library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2601_16536_amd.build` "
                "(there is no CPU or PyTorch fallback)" % LIB_PATH)
        # torch first: it brings its own HIP runtime (same SONAME as ROCm's), and the
        # library must bind to that copy -- two HIP runtimes in one process do not
        # share devices, streams or allocations.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        gemm_args = [vp, vp, vp, vp, ci, ci, ci, ci, vp, vp]
        L.w4a16_gemm.argtypes = gemm_args
        L.w4a16_gemm_ex.argtypes = gemm_args + [ci, ci]
        L.w4a16_gemm_ws.argtypes = gemm_args + [ci, ci, vp, sz]
        L.w4a16_gemm_noalloc.argtypes = gemm_args + [ci, ci]
        L.w4a16_gemm_bf16.argtypes = gemm_args + [ci, ci]
        L.w4a16_set_workspace.argtypes = [vp, sz]
        L.w4a16_tune.argtypes = [ctypes.c_char_p, ci]
        L.w4a16_workspace_bytes.argtypes = [ci, ci, ci, ci]
        L.w4a16_workspace_bytes.restype = sz
        L.w4a16_query_plan.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.POINTER(Plan)]
        L.w4a16_reduce.argtypes = [vp, ci, ci, ci, vp, vp]
        L.w4a16_dequant.argtypes = [vp, vp, vp, ci, ci, ci, vp, vp]
        L.w4a16_quantize.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
        L.w4a16_stream_probe.argtypes = [vp, sz, vp, sz, vp, sz, vp, vp]
        L.w4a16_status_string.argtypes = [ci]
        L.w4a16_status_string.restype = ctypes.c_char_p
        L.w4a16_last_hip_error.argtypes = []
        L.w4a16_last_hip_error.restype = ctypes.c_char_p
        L.w4a16_shutdown.argtypes = []
        L.w4a16_shutdown.restype = None
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().w4a16_status_string(int(status)).decode()


def last_hip_error() -> str:
    return lib().w4a16_last_hip_error().decode()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _check_tensors(X, Wpacked, scales, zeros, group, x_dtype=None):
    """zeros may be None: symmetric quantisation (every zero point is 8, no tensor)."""
    import torch
    for name, t, dt in (("X", X, x_dtype or torch.float16), ("Wpacked", Wpacked, torch.int32),
                        ("scales", scales, torch.float16), ("zeros", zeros, torch.int32)):
        if t is None and name == "zeros":
            continue
        if not t.is_cuda or not t.is_contiguous() or t.dtype != dt:
            raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dt))
    M, K = X.shape
    R, N = Wpacked.shape
    if R * 8 != K or group < 1 or K % group:
        raise ValueError("Wpacked %r does not fit X %r / group %d" % (tuple(Wpacked.shape), tuple(X.shape), group))
    G = K // group
    if tuple(scales.shape) != (G, N) or N % 8 or (zeros is not None and tuple(zeros.shape) != (G, N // 8)):
        raise ValueError("scales/zeros shapes do not fit K=%d N=%d group=%d" % (K, N, group))
    return M, N, K


def raw_gemm(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr) -> int:
    """w4a16_gemm on raw device addresses; returns the status code."""
    return lib().w4a16_gemm(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr)


def raw_gemm_ex(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr, kernel, split) -> int:
    return lib().w4a16_gemm_ex(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr, kernel, split)


def raw_gemm_ws(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr, kernel, split, ws_ptr, ws_bytes) -> int:
    return lib().w4a16_gemm_ws(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr, kernel, split,
                               ws_ptr, ws_bytes)


def raw_gemm_noalloc(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr, kernel=KERNEL_AUTO, split=0) -> int:
    """w4a16_gemm_noalloc on raw device addresses; returns the status code."""
    return lib().w4a16_gemm_noalloc(X_ptr, W_ptr, s_ptr, z_ptr, group, M, N, K, Y_ptr, stream_ptr, kernel, split)


def gemm_noalloc(X, Wpacked, scales, zeros, group: int, out, kernel: int = KERNEL_AUTO, split: int = 0, stream=None):
    """As gemm_ex, through the entry point that allocates nothing: the caller brings Y as well."""
    M, N, K = _check_tensors(X, Wpacked, scales, zeros, group)
    if tuple(out.shape) != (M, N) or not out.is_contiguous():
        raise ValueError("out must be a contiguous [M, N] tensor")
    rc = raw_gemm_noalloc(X.data_ptr(), Wpacked.data_ptr(), scales.data_ptr(), _ptr(zeros), group, M, N, K,
                          out.data_ptr(), _stream(stream), kernel, split)
    if rc:
        raise W4A16Error(rc, "w4a16_gemm_noalloc")
    return out


def set_workspace(workspace) -> None:
    """Registers a caller-owned workspace tensor (uint8, CUDA, 256-byte aligned) for the current device; None removes it.
    The tensor must stay alive while it is registered."""
    if workspace is None:
        rc = lib().w4a16_set_workspace(None, 0)
    else:
        rc = lib().w4a16_set_workspace(workspace.data_ptr(), workspace.numel() * workspace.element_size())
    if rc:
        raise W4A16Error(rc, "w4a16_set_workspace")


def tune(knob: str, value: int) -> None:
    """Sets a tuning knob of the library (sweeps and tests only); 0 restores the scheduler's choice."""
    rc = lib().w4a16_tune(knob.encode(), int(value))
    if rc:
        raise W4A16Error(rc, "w4a16_tune(%r)" % knob)


def gemm(X, Wpacked, scales, zeros, group: int, out=None, stream=None):
    """Y = X * s (W - z) (Eq. 2).  uint32 storage travels as torch.int32 tensors."""
    import torch
    M, N, K = _check_tensors(X, Wpacked, scales, zeros, group)
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = raw_gemm(X.data_ptr(), Wpacked.data_ptr(), scales.data_ptr(), _ptr(zeros), group, M, N, K,
                  Y.data_ptr(), _stream(stream))
    if rc:
        raise W4A16Error(rc, "w4a16_gemm")
    return Y


def gemm_ex(X, Wpacked, scales, zeros, group: int, kernel: int = KERNEL_AUTO, split: int = 0, out=None, stream=None):
    """As gemm, with the kernel family and the split factor S forced (0 / AUTO = scheduler's choice)."""
    import torch
    M, N, K = _check_tensors(X, Wpacked, scales, zeros, group)
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = raw_gemm_ex(X.data_ptr(), Wpacked.data_ptr(), scales.data_ptr(), _ptr(zeros), group, M, N, K,
                     Y.data_ptr(), _stream(stream), kernel, split)
    if rc:
        raise W4A16Error(rc, "w4a16_gemm_ex")
    return Y


def gemm_bf16(X, Wpacked, scales, zeros, group: int, kernel: int = KERNEL_AUTO, split: int = 0, out=None, stream=None):
    """w4a16_gemm_bf16: X and the result are torch.bfloat16; the weights' tensors as in gemm."""
    import torch
    M, N, K = _check_tensors(X, Wpacked, scales, zeros, group, torch.bfloat16)
    Y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    if Y.dtype != torch.bfloat16 or tuple(Y.shape) != (M, N) or not Y.is_contiguous():
        raise ValueError("out must be a contiguous bfloat16 [M, N] tensor")
    rc = lib().w4a16_gemm_bf16(X.data_ptr(), Wpacked.data_ptr(), scales.data_ptr(), _ptr(zeros), group, M, N, K,
                               Y.data_ptr(), _stream(stream), kernel, split)
    if rc:
        raise W4A16Error(rc, "w4a16_gemm_bf16")
    return Y


def gemm_ws(X, Wpacked, scales, zeros, group: int, workspace, kernel: int = KERNEL_AUTO, split: int = 0, out=None,
            stream=None):
    """As gemm_ex, with the caller's workspace tensor (uint8, CUDA, 256-byte aligned)."""
    import torch
    M, N, K = _check_tensors(X, Wpacked, scales, zeros, group)
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = raw_gemm_ws(X.data_ptr(), Wpacked.data_ptr(), scales.data_ptr(), _ptr(zeros), group, M, N, K,
                     Y.data_ptr(), _stream(stream), kernel, split, workspace.data_ptr(),
                     workspace.numel() * workspace.element_size())
    if rc:
        raise W4A16Error(rc, "w4a16_gemm_ws")
    return Y


def workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return int(lib().w4a16_workspace_bytes(M, N, K, group))


def query_plan(M: int, N: int, K: int, group: int, kernel: int = KERNEL_AUTO, split: int = 0) -> dict:
    p = Plan()
    rc = lib().w4a16_query_plan(M, N, K, group, kernel, split, ctypes.byref(p))
    if rc:
        raise W4A16Error(rc, "w4a16_query_plan")
    return p.as_dict()


def reduce(partials, out=None, stream=None):
    """Second pass alone (Algorithm 1, Phase 3): fp32 [S, M, N] -> fp16 [M, N]."""
    import torch
    if not partials.is_cuda or partials.dtype != torch.float32 or not partials.is_contiguous() or partials.dim() != 3:
        raise TypeError("partials must be a contiguous CUDA float32 tensor [S, M, N]")
    S, M, N = partials.shape
    Y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=partials.device)
    rc = lib().w4a16_reduce(partials.data_ptr(), S, M, N, Y.data_ptr(), _stream(stream))
    if rc:
        raise W4A16Error(rc, "w4a16_reduce")
    return Y


def dequant(Wpacked, scales, zeros, group: int, out=None, stream=None):
    """Phase 1 alone (Algorithm 1): the FP16 matrix [K, N] of dequantised weights, for the unfused variant."""
    import torch
    tensors = [Wpacked, scales] + ([zeros] if zeros is not None else [])
    if not all(t.is_cuda for t in tensors):
        raise TypeError("device tensors wanted")
    if Wpacked.dtype != torch.int32 or (zeros is not None and zeros.dtype != torch.int32) or scales.dtype != torch.float16:
        raise TypeError("Wpacked and zeros are int32 (uint32 bits), scales float16")
    if not all(t.is_contiguous() for t in tensors):
        raise TypeError("contiguous tensors wanted")
    K, N = Wpacked.shape[0] * 8, Wpacked.shape[1]
    if K % group or tuple(scales.shape) != (K // group, N) or (zeros is not None and tuple(zeros.shape) != (K // group, N // 8)):
        raise W4A16Error(2, "binding.dequant (shapes of scales / zeros)")
    W16 = out if out is not None else torch.empty((K, N), dtype=torch.float16, device=Wpacked.device)
    rc = lib().w4a16_dequant(Wpacked.data_ptr(), scales.data_ptr(), _ptr(zeros), group, N, K, W16.data_ptr(),
                             _stream(stream))
    if rc:
        raise W4A16Error(rc, "w4a16_dequant")
    return W16


def stream_probe(tensors, sink, stream=None):
    """Measurement aid: reads up to three device tensors once (what a multiply reads: weights, scales, zero points) and
    keeps nothing.  `sink`: a device tensor of at least four bytes."""
    ts = [t for t in tensors if t is not None]
    if not 1 <= len(ts) <= 3 or not all(t.is_cuda and t.is_contiguous() for t in ts) or not sink.is_cuda:
        raise TypeError("one to three contiguous device tensors and a device sink wanted")
    args = []
    for t in ts + [None] * (3 - len(ts)):
        args += [t.data_ptr() if t is not None else None, t.numel() * t.element_size() if t is not None else 0]
    rc = lib().w4a16_stream_probe(*args, sink.data_ptr(), _stream(stream))
    if rc:
        raise W4A16Error(rc, "w4a16_stream_probe")


def quantize(W16, group: int, stream=None):
    """Offline tool (Eq. 1): FP16 weights [K, N] on the GPU -> (Wpacked int32 [K/8, N], scales float16 [G, N],
    zeros int32 [G, N/8]) in the layout gemm reads."""
    import torch
    if not W16.is_cuda or W16.dtype != torch.float16 or not W16.is_contiguous() or W16.dim() != 2:
        raise TypeError("W16 must be a contiguous CUDA float16 matrix [K, N]")
    K, N = W16.shape
    if group < 1 or K % group or K % 8 or N % 8:
        raise W4A16Error(2, "binding.quantize (shape)")
    G = K // group
    Wp = torch.empty((K // 8, N), dtype=torch.int32, device=W16.device)
    s = torch.empty((G, N), dtype=torch.float16, device=W16.device)
    Zp = torch.empty((G, N // 8), dtype=torch.int32, device=W16.device)
    rc = lib().w4a16_quantize(W16.data_ptr(), group, N, K, Wp.data_ptr(), s.data_ptr(), Zp.data_ptr(), _stream(stream))
    if rc:
        raise W4A16Error(rc, "w4a16_quantize")
    return Wp, s, Zp


def shutdown() -> None:
    lib().w4a16_shutdown()


def to_device(X, Wp, scales, Zp, device="cuda"):
    """numpy inputs (float16 / uint32) -> torch tensors on the GPU (uint32 bits as int32)."""
    import numpy as np
    import torch
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    return (t(X).to(device), t(Wp.view(np.int32)).to(device), t(scales).to(device), t(Zp.view(np.int32)).to(device))
