"""ctypes loader for the CPU oracle (``itq3s_ref.c``).

Test infrastructure only: the test-suite, the smoke check and the benchmark's cpu_baseline leg
use it; the product (``paper_2603_27914_amd``) never imports this module.  Host numpy arrays in,
host numpy arrays out; everything the oracle computes is fp64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# (the mutation test of the pins points these at a deliberately broken copy of the source)
_SRC = os.environ.get("ITQ3S_REF_SRC", os.path.join(_HERE, "itq3s_ref.c"))
_LIB = os.environ.get("ITQ3S_REF_LIB", os.path.join(_HERE, "libitq3s_ref.so"))

FLAG_NONFINITE, FLAG_SCALE_SAT, FLAG_Z_CLAMP, FLAG_BAD_CODE = 1, 2, 4, 8


def build(force=False):
    """Compile the oracle with gcc (contraction off: every fp64 operation rounds once)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, vp, u32p = ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p
        L.itq3s_ref_codes_bytes.restype = ctypes.c_size_t
        L.itq3s_ref_codes_bytes.argtypes = [i64, i64]
        L.itq3s_ref_scales_bytes.restype = ctypes.c_size_t
        L.itq3s_ref_scales_bytes.argtypes = [i64, i64]
        L.itq3s_ref_quantize.argtypes = [vp, i64, i64, i64, u32p, u32p, u32p]
        L.itq3s_ref_dequantize.argtypes = [u32p, u32p, i64, i64, vp, i64, u32p]
        L.itq3s_ref_matmul.argtypes = [u32p, u32p, i64, i64, vp, i64, i64, vp, i64]
        L.itq3s_ref_matmul_rows.argtypes = [u32p, u32p, i64, i64, vp, i64, i64, vp, i64, i64, i64]
        L.itq3s_ref_roundtrip_n.argtypes = [vp, i64, i64, i64, ctypes.c_int, vp, u32p, vp, u32p]
        L.itq3s_ref_subscales_bytes.restype = ctypes.c_size_t
        L.itq3s_ref_subscales_bytes.argtypes = [i64, i64]
        L.itq3s_ref_quantize_sub.argtypes = [vp, i64, i64, i64, u32p, u32p, u32p, u32p]
        L.itq3s_ref_dequantize_sub.argtypes = [u32p, u32p, u32p, i64, i64, vp, i64, u32p]
        L.itq3s_ref_matmul_sub_rows.argtypes = [u32p, u32p, u32p, i64, i64, vp, i64, i64, vp, i64, i64, i64]
        L.itq3s_ref_quantize_block_sub.argtypes = [vp, vp, vp, u32p]
        L.itq3s_ref_quantize_block_sub.restype = ctypes.c_uint32
        L.itq3s_ref_fwht256.argtypes = [vp]
        L.itq3s_ref_fwht256.restype = None
        L.itq3s_ref_forward_block.argtypes = [vp, vp]
        L.itq3s_ref_forward_block.restype = None
        L.itq3s_ref_quantize_block.argtypes = [vp, vp, u32p]
        L.itq3s_ref_quantize_block.restype = ctypes.c_uint32
        L.itq3s_ref_f32_to_f16.argtypes = [ctypes.c_float]
        L.itq3s_ref_f32_to_f16.restype = ctypes.c_uint16
        L.itq3s_ref_f16_to_f64.argtypes = [ctypes.c_uint16]
        L.itq3s_ref_f16_to_f64.restype = ctypes.c_double
        L.itq3s_ref_t_star.restype = ctypes.c_double
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(status):
    if status != 0:
        raise ValueError("oracle rejected the arguments (status %d)" % status)


def codes_words(N, K):
    return lib().itq3s_ref_codes_bytes(N, K) // 4


def scales_words(N, K):
    return lib().itq3s_ref_scales_bytes(N, K) // 4


def fwht256(a):
    """Unnormalised 256-point butterfly network on a copy of ``a`` (fp64)."""
    out = np.ascontiguousarray(a, dtype=np.float64).copy()
    assert out.shape == (256,)
    lib().itq3s_ref_fwht256(_ptr(out))
    return out


def forward_block(w):
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.shape == (256,)
    out = np.empty(256, dtype=np.float64)
    lib().itq3s_ref_forward_block(_ptr(w), _ptr(out))
    return out


def quantize_block(w):
    """-> (codes uint8[256] in {0,1,2}, scale word, flags)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.shape == (256,)
    codes = np.empty(256, dtype=np.uint8)
    flags = np.zeros(1, dtype=np.uint32)
    word = lib().itq3s_ref_quantize_block(_ptr(w), _ptr(codes), _ptr(flags))
    return codes, int(word), int(flags[0])


def quantize(W):
    """W fp32 [N, K] -> (codes uint32, scales uint32, flags)."""
    W = np.asarray(W)
    assert W.dtype == np.float32 and W.ndim == 2 and W.strides[1] == 4
    N, K = W.shape
    codes = np.zeros(codes_words(N, K), dtype=np.uint32)
    scales = np.zeros(scales_words(N, K), dtype=np.uint32)
    flags = np.zeros(1, dtype=np.uint32)
    _check(lib().itq3s_ref_quantize(_ptr(W), N, K, W.strides[0] // 4, _ptr(codes), _ptr(scales), _ptr(flags)))
    return codes, scales, int(flags[0])


def roundtrip_n(W, n):
    """Block-size ablation: quantize and reconstruct W fp32 [N, K] with blocks of n channels.
    -> (codes uint8 [N, K], scale words uint32 [N, K/n], W_hat fp64 [N, K], flags)."""
    W = np.asarray(W)
    assert W.dtype == np.float32 and W.ndim == 2 and W.strides[1] == 4
    N, K = W.shape
    codes = np.zeros((N, K), dtype=np.uint8)
    scales = np.zeros((N, K // n), dtype=np.uint32)
    what = np.zeros((N, K), dtype=np.float64)
    flags = np.zeros(1, dtype=np.uint32)
    _check(lib().itq3s_ref_roundtrip_n(_ptr(W), N, K, W.strides[0] // 4, n, _ptr(codes), _ptr(scales), _ptr(what), _ptr(flags)))
    return codes, scales, what, int(flags[0])


def dequantize(codes, scales, N, K, return_flags=False):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    scales = np.ascontiguousarray(scales, dtype=np.uint32)
    assert codes.size == codes_words(N, K) and scales.size == scales_words(N, K)
    out = np.empty((N, K), dtype=np.float64)
    flags = np.zeros(1, dtype=np.uint32)
    _check(lib().itq3s_ref_dequantize(_ptr(codes), _ptr(scales), N, K, _ptr(out), K, _ptr(flags)))
    return (out, int(flags[0])) if return_flags else out


def matmul(codes, scales, N, K, X, rows=None):
    """X: float16 [M, K].  -> Y fp64 [M, N]; with rows=(n0, n1) only those columns are filled."""
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    scales = np.ascontiguousarray(scales, dtype=np.uint32)
    X = np.ascontiguousarray(X)
    assert X.dtype == np.float16 and X.ndim == 2 and X.shape[1] == K
    assert codes.size == codes_words(N, K) and scales.size == scales_words(N, K)
    M = X.shape[0]
    Y = np.zeros((M, N), dtype=np.float64)
    n0, n1 = (0, N) if rows is None else rows
    _check(lib().itq3s_ref_matmul_rows(_ptr(codes), _ptr(scales), N, K, _ptr(X), M, K, _ptr(Y), N, n0, n1))
    return Y


def f32_to_f16_bits(x):
    return int(lib().itq3s_ref_f32_to_f16(ctypes.c_float(x)))


def f16_bits_to_f64(h):
    return float(lib().itq3s_ref_f16_to_f64(ctypes.c_uint16(h)))


def t_star():
    return float(lib().itq3s_ref_t_star())


# ---- sub-block-scale variant (116 bytes per block)


def subscales_words(N, K):
    return lib().itq3s_ref_subscales_bytes(N, K) // 4


def quantize_block_sub(w):
    """-> (codes uint8[256], scale word, sub-scale bit patterns uint16[8], flags)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.shape == (256,)
    codes = np.empty(256, dtype=np.uint8)
    subs = np.zeros(8, dtype=np.uint16)
    flags = np.zeros(1, dtype=np.uint32)
    word = lib().itq3s_ref_quantize_block_sub(_ptr(w), _ptr(codes), _ptr(subs), _ptr(flags))
    return codes, int(word), subs, int(flags[0])


def quantize_sub(W):
    """W fp32 [N, K] -> (codes uint32, scales uint32, subscales uint32, flags)."""
    W = np.asarray(W)
    assert W.dtype == np.float32 and W.ndim == 2 and W.strides[1] == 4
    N, K = W.shape
    codes = np.zeros(codes_words(N, K), dtype=np.uint32)
    scales = np.zeros(scales_words(N, K), dtype=np.uint32)
    subs = np.zeros(subscales_words(N, K), dtype=np.uint32)
    flags = np.zeros(1, dtype=np.uint32)
    _check(lib().itq3s_ref_quantize_sub(_ptr(W), N, K, W.strides[0] // 4, _ptr(codes), _ptr(scales), _ptr(subs), _ptr(flags)))
    return codes, scales, subs, int(flags[0])


def dequantize_sub(codes, scales, subs, N, K, return_flags=False):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    scales = np.ascontiguousarray(scales, dtype=np.uint32)
    subs = np.ascontiguousarray(subs, dtype=np.uint32)
    assert codes.size == codes_words(N, K) and scales.size == scales_words(N, K) and subs.size == subscales_words(N, K)
    out = np.empty((N, K), dtype=np.float64)
    flags = np.zeros(1, dtype=np.uint32)
    _check(lib().itq3s_ref_dequantize_sub(_ptr(codes), _ptr(scales), _ptr(subs), N, K, _ptr(out), K, _ptr(flags)))
    return (out, int(flags[0])) if return_flags else out


def matmul_sub(codes, scales, subs, N, K, X, rows=None):
    codes = np.ascontiguousarray(codes, dtype=np.uint32)
    scales = np.ascontiguousarray(scales, dtype=np.uint32)
    subs = np.ascontiguousarray(subs, dtype=np.uint32)
    X = np.ascontiguousarray(X)
    assert X.dtype == np.float16 and X.ndim == 2 and X.shape[1] == K
    assert codes.size == codes_words(N, K) and scales.size == scales_words(N, K) and subs.size == subscales_words(N, K)
    M = X.shape[0]
    Y = np.zeros((M, N), dtype=np.float64)
    n0, n1 = (0, N) if rows is None else rows
    _check(lib().itq3s_ref_matmul_sub_rows(_ptr(codes), _ptr(scales), _ptr(subs), N, K, _ptr(X), M, K, _ptr(Y), N, n0, n1))
    return Y
