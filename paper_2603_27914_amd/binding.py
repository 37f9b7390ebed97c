"""Thin ctypes binding over libitq3s (the C ABI declared in include/itq3s.h).

Argument marshalling only: torch tensors supply device memory and the current HIP stream; every
step of the computation runs in the library's kernels.  There is no CPU fallback -- if the shared
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libitq3s.so")

F32, F16 = 0, 1
FLAG_NONFINITE, FLAG_SCALE_SAT, FLAG_Z_CLAMP, FLAG_BAD_CODE, FLAG_ACT_RANGE = 1, 2, 4, 8, 16

EXPORTS = [
    "itq3s_codes_bytes",
    "itq3s_scales_bytes",
    "itq3s_matmul_workspace_bytes",
    "itq3s_quantize",
    "itq3s_dequantize",
    "itq3s_roundtrip",
    "itq3s_matmul",
    "itq3s_matmul_grouped",
    "itq3s_matmul_static",
    "itq3s_subscales_bytes",
    "itq3s_quantize_sub",
    "itq3s_dequantize_sub",
    "itq3s_matmul_sub",
    "itq3s_matmul_grouped_timed",
    "itq3s_matmul_timed",
    "itq3s_matmul_weight_side",
    "itq3s_matmul_weight_side_timed",
    "itq3s_read_probe",
    "itq3s_strerror",
    "itq3s_version",
]

MAX_GROUP = 4


class Weight(ctypes.Structure):
    """struct itq3s_weight"""

    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("N", ctypes.c_int64), ("Y", ctypes.c_void_p), ("ldy", ctypes.c_int64)]


_lib = None


class Itq3sError(RuntimeError):
    pass


def lib():
    """Load libitq3s.so (built by ``paper_2603_27914_amd.build`` / ``__graft_entry__.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise Itq3sError("libitq3s.so is not built: run `python -m paper_2603_27914_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        i64, vp, sz, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.itq3s_codes_bytes.restype = sz
        L.itq3s_codes_bytes.argtypes = [i64, i64]
        L.itq3s_scales_bytes.restype = sz
        L.itq3s_scales_bytes.argtypes = [i64, i64]
        L.itq3s_matmul_workspace_bytes.restype = sz
        L.itq3s_matmul_workspace_bytes.argtypes = [i64, i64, i64]
        L.itq3s_quantize.restype = ci
        L.itq3s_quantize.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp]
        L.itq3s_dequantize.restype = ci
        L.itq3s_dequantize.argtypes = [vp, vp, i64, i64, vp, ci, i64, vp, vp]
        L.itq3s_roundtrip.restype = ci
        L.itq3s_roundtrip.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp, i64, vp, vp, vp]
        L.itq3s_matmul.restype = ci
        L.itq3s_matmul.argtypes = [vp, vp, i64, i64, vp, i64, i64, vp, ci, i64, vp, sz, vp, vp]
        L.itq3s_subscales_bytes.restype = sz
        L.itq3s_subscales_bytes.argtypes = [i64, i64]
        L.itq3s_quantize_sub.restype = ci
        L.itq3s_quantize_sub.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp]
        L.itq3s_dequantize_sub.restype = ci
        L.itq3s_dequantize_sub.argtypes = [vp, vp, vp, i64, i64, vp, ci, i64, vp, vp]
        L.itq3s_matmul_sub.restype = ci
        L.itq3s_matmul_sub.argtypes = [vp, vp, vp, i64, i64, vp, i64, i64, vp, ci, i64, vp, sz, vp, vp]
        L.itq3s_matmul_static.restype = ci
        L.itq3s_matmul_static.argtypes = [vp, vp, i64, i64, vp, i64, i64, vp, ci, i64, vp, vp]
        L.itq3s_matmul_grouped.restype = ci
        L.itq3s_matmul_grouped.argtypes = [ctypes.POINTER(Weight), ci, i64, vp, i64, i64, ci, vp, sz, vp, vp]
        L.itq3s_matmul_grouped_timed.restype = ci
        L.itq3s_matmul_grouped_timed.argtypes = L.itq3s_matmul_grouped.argtypes + [ctypes.POINTER(ctypes.c_float)]
        L.itq3s_matmul_timed.restype = ci
        L.itq3s_matmul_timed.argtypes = L.itq3s_matmul.argtypes + [ctypes.POINTER(ctypes.c_float)]
        L.itq3s_matmul_weight_side.restype = ci
        L.itq3s_matmul_weight_side.argtypes = [vp, vp, i64, i64, vp, i64, i64, vp, ci, i64, vp, vp]
        L.itq3s_matmul_weight_side_timed.restype = ci
        L.itq3s_matmul_weight_side_timed.argtypes = L.itq3s_matmul_weight_side.argtypes + [ctypes.POINTER(ctypes.c_float)]
        L.itq3s_read_probe.restype = ci
        L.itq3s_read_probe.argtypes = [vp, sz, vp, vp]
        L.itq3s_strerror.restype = ctypes.c_char_p
        L.itq3s_strerror.argtypes = [ci]
        L.itq3s_version.restype = ci
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise Itq3sError("libitq3s: %s (status %d)" % (lib().itq3s_strerror(status).decode(), status))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _need_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise Itq3sError("libitq3s works on device memory only; got a CPU tensor")


def _need_packed(codes, scales, N, K, *others):
    """The C ABI sees pointers, not sizes: refuse here what would make a kernel read outside the
    packed arrays (a wrong N or K, a slice, a tensor of another type or on another device)."""
    cb, sb = itq3s_codes_bytes(N, K), itq3s_scales_bytes(N, K)
    if cb == 0:
        raise Itq3sError("bad shape: N and K must be positive, K a multiple of 256")
    for name, t, nbytes in (("codes", codes, cb), ("scales", scales, sb)):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise Itq3sError("%s must be a contiguous int32 tensor" % name)
        if t.numel() * 4 < nbytes:
            raise Itq3sError("%s holds %d bytes, W[%d, %d] needs %d" % (name, t.numel() * 4, N, K, nbytes))
        if t.device != codes.device:
            raise Itq3sError("codes and scales must be on the same device")
    for t in others:
        if t is not None and t.device != codes.device:
            raise Itq3sError("every tensor of a call must be on the same device")


def _need_flags(status_flags):
    if status_flags is not None and (status_flags.dtype != torch.int32 or status_flags.numel() < 1 or not status_flags.is_contiguous()):
        raise Itq3sError("status_flags must be a contiguous int32 tensor with at least one element")


def itq3s_codes_bytes(N, K):
    return lib().itq3s_codes_bytes(N, K)


def itq3s_scales_bytes(N, K):
    return lib().itq3s_scales_bytes(N, K)


def itq3s_matmul_workspace_bytes(M, N, K):
    return lib().itq3s_matmul_workspace_bytes(M, N, K)


def itq3s_version():
    return lib().itq3s_version()


def alloc_packed(N, K, device="cuda"):
    """Uninitialised (codes int32[...], scales int32[...]) tensors of the right size."""
    cb, sb = itq3s_codes_bytes(N, K), itq3s_scales_bytes(N, K)
    if cb == 0:
        raise Itq3sError("bad shape: K must be a positive multiple of 256")
    return torch.empty(cb // 4, dtype=torch.int32, device=device), torch.empty(sb // 4, dtype=torch.int32, device=device)


def itq3s_quantize(W, codes=None, scales=None, status_flags=None):
    """W: float32 [N, K] device tensor (row stride arbitrary) -> (codes, scales) int32 device tensors."""
    _need_cuda(W, codes, scales, status_flags)
    if W.dtype != torch.float32 or W.dim() != 2 or W.stride(1) != 1:
        raise Itq3sError("W must be float32 [N, K] with unit column stride")
    N, K = W.shape
    if codes is None or scales is None:
        codes, scales = alloc_packed(N, K, W.device)
    _need_packed(codes, scales, N, K, W, status_flags)
    _need_flags(status_flags)
    _check(lib().itq3s_quantize(_ptr(W), N, K, W.stride(0), _ptr(codes), _ptr(scales), _ptr(status_flags), _stream()))
    return codes, scales


def itq3s_dequantize(codes, scales, N, K, out=None, dtype=torch.float32, status_flags=None):
    """-> reconstructed weights [N, K] (float32 or float16) on the device."""
    _need_cuda(codes, scales, out, status_flags)
    _need_packed(codes, scales, N, K, out, status_flags)
    _need_flags(status_flags)
    if out is None:
        out = torch.empty((N, K), dtype=dtype, device=codes.device)
    if out.dtype not in (torch.float32, torch.float16) or out.dim() != 2 or out.stride(1) != 1 or tuple(out.shape) != (N, K):
        raise Itq3sError("out must be float32/float16 [N, K] with unit column stride")
    _check(
        lib().itq3s_dequantize(
            _ptr(codes), _ptr(scales), N, K, _ptr(out), F16 if out.dtype == torch.float16 else F32, out.stride(0), _ptr(status_flags), _stream()
        )
    )
    return out


def itq3s_roundtrip(W, block_size, codes=True, scales=True, w_hat=True, err2=None, status_flags=None):
    """Rotate - quantize - reconstruct with transform length block_size (32 .. 512), unpacked.

    W: float32 [N, K] device tensor.  codes / scales / w_hat: True to allocate, False to skip, or a
    tensor to fill (uint8 [N, K], int32 [N, K/block_size], float32 [N, K]).  err2: float64[2] device
    tensor the call adds (sum of squared errors, sum of squared weights) to, or None.
    -> (codes, scales, w_hat), None where skipped."""
    _need_cuda(W, err2, status_flags)
    if W.dtype != torch.float32 or W.dim() != 2 or W.stride(1) != 1:
        raise Itq3sError("W must be float32 [N, K] with unit column stride")
    N, K = W.shape
    if block_size <= 0 or K % block_size != 0:
        raise Itq3sError("K must be a multiple of block_size")

    def want(arg, shape, dtype):
        if arg is True:
            return torch.empty(shape, dtype=dtype, device=W.device)
        if arg is False or arg is None:
            return None
        _need_cuda(arg)
        if arg.dtype != dtype or tuple(arg.shape) != shape or arg.stride(-1) != 1:
            raise Itq3sError("output tensor must be %s %s with unit column stride" % (dtype, shape))
        return arg

    codes = want(codes, (N, K), torch.uint8)
    scales = want(scales, (N, K // block_size), torch.int32)
    w_hat = want(w_hat, (N, K), torch.float32)
    if (codes is not None and not codes.is_contiguous()) or (scales is not None and not scales.is_contiguous()):
        raise Itq3sError("codes and scales must be contiguous")
    if err2 is not None and (err2.dtype != torch.float64 or err2.numel() != 2 or not err2.is_contiguous()):
        raise Itq3sError("err2 must be a contiguous float64[2] tensor")
    _check(
        lib().itq3s_roundtrip(
            _ptr(W), N, K, W.stride(0), block_size, _ptr(codes), _ptr(scales), _ptr(w_hat), w_hat.stride(0) if w_hat is not None else 0,
            _ptr(err2), _ptr(status_flags), _stream()
        )
    )
    return codes, scales, w_hat


def itq3s_matmul_weight_side(codes, scales, N, K, X, out=None, dtype=torch.float32, status_flags=None, timed=False):
    """Y = X @ W_hat^T with the inverse transform inside the weight tile loader (the paper's placement).
    timed=True waits and returns (Y, kernel milliseconds)."""
    _need_cuda(codes, scales, X, out, status_flags)
    _need_packed(codes, scales, N, K, X, out, status_flags)
    _need_flags(status_flags)
    if X.dtype != torch.float16 or X.dim() != 2 or X.stride(1) != 1 or X.shape[1] != K:
        raise Itq3sError("X must be float16 [M, K] with unit column stride")
    M = X.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=X.device)
    if out.dtype not in (torch.float32, torch.float16) or out.dim() != 2 or out.stride(1) != 1 or tuple(out.shape) != (M, N):
        raise Itq3sError("out must be float32/float16 [M, N] with unit column stride")
    ms = ctypes.c_float(0.0)
    args = (_ptr(codes), _ptr(scales), N, K, _ptr(X), M, X.stride(0), _ptr(out), F16 if out.dtype == torch.float16 else F32,
            out.stride(0), _ptr(status_flags), _stream())
    if timed:
        _check(lib().itq3s_matmul_weight_side_timed(*args, ctypes.byref(ms)))
        return out, float(ms.value)
    _check(lib().itq3s_matmul_weight_side(*args))
    return out


def itq3s_matmul_weight_side_timed(codes, scales, N, K, X, out=None, dtype=torch.float32, status_flags=None):
    """itq3s_matmul_weight_side, then wait; -> (Y, milliseconds the kernel ran by the GPU's clock)."""
    return itq3s_matmul_weight_side(codes, scales, N, K, X, out, dtype, status_flags, timed=True)


def itq3s_read_probe(buf, sink):
    """Plain streaming read of a device tensor (measurement aid); sink: int32[1] device tensor."""
    _need_cuda(buf, sink)
    _check(lib().itq3s_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()))


def itq3s_matmul_grouped_timed(weights, K, X, outs=None, dtype=torch.float32, workspace=None, status_flags=None):
    """itq3s_matmul_grouped, then wait; -> (outs, milliseconds the contraction kernel ran by the GPU's clock)."""
    ms = ctypes.c_float(0.0)
    outs = itq3s_matmul_grouped(weights, K, X, outs, dtype, workspace, status_flags, _timed=ms)
    return outs, float(ms.value)


def itq3s_matmul_grouped(weights, K, X, outs=None, dtype=torch.float32, workspace=None, status_flags=None, _timed=None):
    """weights: list of (codes, scales, N) sharing K -> list of Y_t[M, N_t] = X @ W_hat_t^T, one call."""
    _need_cuda(X, workspace, status_flags)
    M = X.shape[0]
    if X.dtype != torch.float16 or X.dim() != 2 or X.stride(1) != 1 or X.shape[1] != K:
        raise Itq3sError("X must be float16 [M, K] with unit column stride")
    if not 1 <= len(weights) <= MAX_GROUP:
        raise Itq3sError("1..%d tensors per grouped call" % MAX_GROUP)
    if outs is None:
        outs = [torch.empty((M, N), dtype=dtype, device=X.device) for _, _, N in weights]
    if len(outs) != len(weights) or len({o.dtype for o in outs}) != 1 or outs[0].dtype not in (torch.float32, torch.float16):
        raise Itq3sError("outs: one float32/float16 tensor per weight tensor, all of one dtype")
    _need_flags(status_flags)
    arr = (Weight * len(weights))()
    for i, ((codes, scales, N), out) in enumerate(zip(weights, outs)):
        _need_cuda(codes, scales, out)
        _need_packed(codes, scales, N, K, X, out, workspace, status_flags)
        if out.dim() != 2 or out.stride(1) != 1 or tuple(out.shape) != (M, N):
            raise Itq3sError("out %d must be [M, N] with unit column stride" % i)
        arr[i] = Weight(codes.data_ptr(), scales.data_ptr(), N, out.data_ptr(), out.stride(0))
    _need_cuda(X, workspace, status_flags)
    if workspace is None:
        workspace = torch.empty(max(itq3s_matmul_workspace_bytes(M, N, K) for _, _, N in weights), dtype=torch.uint8, device=X.device)
    args = (
        arr, len(weights), K, _ptr(X), M, X.stride(0), F16 if outs[0].dtype == torch.float16 else F32,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(status_flags), _stream(),
    )
    if _timed is None:
        _check(lib().itq3s_matmul_grouped(*args))
    else:
        _check(lib().itq3s_matmul_grouped_timed(*args, ctypes.byref(_timed)))
    return outs


def itq3s_matmul_static(codes, scales, N, K, X, out, status_flags=None):
    """itq3s_matmul with the scratch in the library's static device array: nothing is allocated, so
    `out` (float32/float16 [M, N]) must be given."""
    _need_cuda(codes, scales, X, out, status_flags)
    _need_packed(codes, scales, N, K, X, out, status_flags)
    _need_flags(status_flags)
    if X.dtype != torch.float16 or X.dim() != 2 or X.stride(1) != 1 or X.shape[1] != K:
        raise Itq3sError("X must be float16 [M, K] with unit column stride")
    M = X.shape[0]
    if out.dtype not in (torch.float32, torch.float16) or out.dim() != 2 or out.stride(1) != 1 or tuple(out.shape) != (M, N):
        raise Itq3sError("out must be float32/float16 [M, N] with unit column stride")
    _check(lib().itq3s_matmul_static(_ptr(codes), _ptr(scales), N, K, _ptr(X), M, X.stride(0), _ptr(out), F16 if out.dtype == torch.float16 else F32,
                                     out.stride(0), _ptr(status_flags), _stream()))
    return out


def itq3s_matmul_timed(codes, scales, N, K, X, out=None, dtype=torch.float32, workspace=None, status_flags=None):
    """itq3s_matmul, then wait; -> (Y, milliseconds the contraction kernel ran by the GPU's clock)."""
    ms = ctypes.c_float(0.0)
    out = itq3s_matmul(codes, scales, N, K, X, out, dtype, workspace, status_flags, _timed=ms)
    return out, float(ms.value)


def itq3s_matmul(codes, scales, N, K, X, out=None, dtype=torch.float32, workspace=None, status_flags=None, _timed=None):
    """Y[M, N] = X[M, K] @ W_hat[N, K]^T from the packed weights.  X: float16 device tensor."""
    _need_cuda(codes, scales, X, out, workspace, status_flags)
    _need_packed(codes, scales, N, K, X, out, workspace, status_flags)
    _need_flags(status_flags)
    if X.dtype != torch.float16 or X.dim() != 2 or X.stride(1) != 1 or X.shape[1] != K:
        raise Itq3sError("X must be float16 [M, K] with unit column stride")
    M = X.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=X.device)
    if out.dtype not in (torch.float32, torch.float16) or out.dim() != 2 or out.stride(1) != 1 or tuple(out.shape) != (M, N):
        raise Itq3sError("out must be float32/float16 [M, N] with unit column stride")
    need = itq3s_matmul_workspace_bytes(M, N, K)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    args = (
        _ptr(codes), _ptr(scales), N, K, _ptr(X), M, X.stride(0), _ptr(out), F16 if out.dtype == torch.float16 else F32,
        out.stride(0), _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(status_flags), _stream(),
    )
    if _timed is None:
        _check(lib().itq3s_matmul(*args))
    else:
        _check(lib().itq3s_matmul_timed(*args, ctypes.byref(_timed)))
    return out


# ---- the sub-block-scale variant of the format (116 bytes per block)


def itq3s_subscales_bytes(N, K):
    return lib().itq3s_subscales_bytes(N, K)


def _need_subscales(subscales, codes, N, K):
    nbytes = itq3s_subscales_bytes(N, K)
    if subscales.dtype != torch.int32 or not subscales.is_contiguous() or subscales.numel() * 4 < nbytes or subscales.device != codes.device:
        raise Itq3sError("subscales must be a contiguous int32 tensor of at least %d bytes on the device of codes" % nbytes)


def itq3s_quantize_sub(W, out=None, status_flags=None):
    """W: float32 [N, K] device tensor -> (codes, scales, subscales) int32 device tensors
    (written into `out`, a triple from an earlier call on the same shape, if given)."""
    _need_cuda(W, status_flags)
    _need_flags(status_flags)
    if W.dtype != torch.float32 or W.dim() != 2 or W.stride(1) != 1:
        raise Itq3sError("W must be float32 [N, K] with unit column stride")
    N, K = W.shape
    if out is not None:
        codes, scales, subscales = out
        _need_cuda(codes, scales, subscales)
        _need_packed(codes, scales, N, K, subscales)
        _need_subscales(subscales, codes, N, K)
    else:
        codes, scales = alloc_packed(N, K, W.device)
        subscales = torch.empty(itq3s_subscales_bytes(N, K) // 4, dtype=torch.int32, device=W.device)
    _check(lib().itq3s_quantize_sub(_ptr(W), N, K, W.stride(0), _ptr(codes), _ptr(scales), _ptr(subscales), _ptr(status_flags), _stream()))
    return codes, scales, subscales


def itq3s_dequantize_sub(codes, scales, subscales, N, K, dtype=torch.float32, status_flags=None):
    _need_cuda(codes, scales, subscales, status_flags)
    _need_packed(codes, scales, N, K, subscales, status_flags)
    _need_subscales(subscales, codes, N, K)
    _need_flags(status_flags)
    if dtype not in (torch.float32, torch.float16):
        raise Itq3sError("dtype must be float32 or float16")
    out = torch.empty((N, K), dtype=dtype, device=codes.device)
    _check(lib().itq3s_dequantize_sub(_ptr(codes), _ptr(scales), _ptr(subscales), N, K, _ptr(out), F16 if dtype == torch.float16 else F32, out.stride(0),
                                      _ptr(status_flags), _stream()))
    return out


def itq3s_matmul_sub(codes, scales, subscales, N, K, X, dtype=torch.float32, out=None, workspace=None, status_flags=None):
    """Y[M, N] = X[M, K] @ W_hat[N, K]^T from weights packed in the sub-block-scale variant.
    workspace: uint8 tensor of itq3s_matmul_workspace_bytes(min(M, 16), N, K) bytes for 5 <= M <= 64
    (allocated here if not given)."""
    _need_cuda(codes, scales, subscales, X, status_flags, workspace)
    _need_packed(codes, scales, N, K, subscales, X, status_flags)
    _need_subscales(subscales, codes, N, K)
    _need_flags(status_flags)
    if X.dtype != torch.float16 or X.dim() != 2 or X.stride(1) != 1 or X.shape[1] != K:
        raise Itq3sError("X must be float16 [M, K] with unit column stride")
    if dtype not in (torch.float32, torch.float16):
        raise Itq3sError("dtype must be float32 or float16")
    M = X.shape[0]
    if workspace is None and 4 < M <= 64:
        workspace = torch.empty(itq3s_matmul_workspace_bytes(min(M, 16), N, K), dtype=torch.uint8, device=X.device)
    if workspace is not None and (workspace.dtype != torch.uint8 or not workspace.is_contiguous()):
        raise Itq3sError("workspace must be a contiguous uint8 tensor")
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=X.device)
    elif not out.is_cuda or out.dtype not in (torch.float32, torch.float16) or tuple(out.shape) != (M, N) or out.stride(1) != 1:
        raise Itq3sError("out must be a float32 or float16 [M, N] device tensor with unit column stride")
    else:
        dtype = out.dtype
    _check(lib().itq3s_matmul_sub(_ptr(codes), _ptr(scales), _ptr(subscales), N, K, _ptr(X), M, X.stride(0), _ptr(out), F16 if dtype == torch.float16 else F32,
                                  out.stride(0), _ptr(workspace), workspace.numel() if workspace is not None else 0, _ptr(status_flags), _stream()))
    return out
