"""ctypes/numpy front end of the C oracle (test infrastructure only; see fp6_oracle.c).

All fp16 data cross this interface as numpy uint16 bit patterns or numpy float16
arrays (viewed, never converted).  Nothing here does arithmetic of the method: it
marshals arrays into the C functions.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        L.fp6o_half_to_double.restype = ctypes.c_double
        L.fp6o_half_to_double.argtypes = [ctypes.c_uint16]
        L.fp6o_round_ratio_to_half.restype = ctypes.c_uint16
        L.fp6o_round_ratio_to_half.argtypes = [i64, i64]
        L.fp6o_e3m2_value.restype = ctypes.c_double
        L.fp6o_e3m2_value.argtypes = [ctypes.c_int]
        L.fp6o_bias_shift_bits.restype = ctypes.c_uint16
        L.fp6o_bias_shift_bits.argtypes = [ctypes.c_int]
        L.fp6o_row_scale.restype = ctypes.c_int
        L.fp6o_row_scale.argtypes = [p, i64, p]
        L.fp6o_quantize.restype = ctypes.c_int
        L.fp6o_quantize.argtypes = [p, i64, i64, p, p]
        L.fp6o_split42.restype = None
        L.fp6o_split42.argtypes = [p, i64, p, p]
        L.fp6o_join42.restype = None
        L.fp6o_join42.argtypes = [p, p, i64, p]
        L.fp6o_dequantize.restype = None
        L.fp6o_dequantize.argtypes = [p, p, i64, i64, p]
        L.fp6o_linear.restype = None
        L.fp6o_linear.argtypes = [p, i64, p, p, i64, i64, p]
        L.fp6o_quantize_fgq.restype = ctypes.c_int
        L.fp6o_quantize_fgq.argtypes = [p, i64, i64, i64, p, p]
        L.fp6o_dequantize_fgq.restype = None
        L.fp6o_dequantize_fgq.argtypes = [p, p, i64, i64, i64, p]
        L.fp6o_linear_bf16.restype = None
        L.fp6o_linear_bf16.argtypes = [p, i64, p, p, i64, i64, p]
        L.fp6o_bf16_to_double.restype = ctypes.c_double
        L.fp6o_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.fp6o_double_to_bf16.restype = ctypes.c_uint16
        L.fp6o_double_to_bf16.argtypes = [ctypes.c_double]
        L.fp6o_linear_fgq.restype = None
        L.fp6o_linear_fgq.argtypes = [p, i64, p, p, i64, i64, i64, p]
        L.fp5o_e3m1_value.restype = ctypes.c_double
        L.fp5o_e3m1_value.argtypes = [ctypes.c_int]
        L.fp5o_bias_shift_bits.restype = ctypes.c_uint16
        L.fp5o_bias_shift_bits.argtypes = [ctypes.c_int]
        L.fp5o_quantize.restype = ctypes.c_int
        L.fp5o_quantize.argtypes = [p, i64, i64, p, p]
        L.fp5o_split41.restype = None
        L.fp5o_split41.argtypes = [p, i64, p, p]
        L.fp5o_dequantize.restype = None
        L.fp5o_dequantize.argtypes = [p, p, i64, i64, p]
        L.fp5o_linear.restype = None
        L.fp5o_linear.argtypes = [p, i64, p, p, i64, i64, p]
        L.fp6o_threads.restype = ctypes.c_int
        L.fp6o_threads.argtypes = []
        _LIB = L
    return _LIB


def _bits(a) -> np.ndarray:
    """fp16 array (float16 or uint16 bits) -> contiguous uint16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("expected float16 or uint16 (fp16 bit patterns), got %s" % a.dtype)
    return np.ascontiguousarray(a)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(lib().fp6o_threads())


def half_to_double(bits: int) -> float:
    return float(lib().fp6o_half_to_double(int(bits)))


def round_ratio_to_half(num: int, den: int) -> int:
    return int(lib().fp6o_round_ratio_to_half(int(num), int(den)))


def e3m2_value(code: int) -> float:
    return float(lib().fp6o_e3m2_value(int(code)))


def bias_shift_bits(code: int) -> int:
    return int(lib().fp6o_bias_shift_bits(int(code)))


def row_scale(w) -> int:
    w = _bits(w).reshape(-1)
    out = np.zeros(1, np.uint16)
    st = lib().fp6o_row_scale(_ptr(w), w.size, _ptr(out))
    if st != 0:
        raise ValueError("oracle: non-finite weight (status %d)" % st)
    return int(out[0])


def quantize(W):
    """W fp16 [N,K] -> (codes uint8 [N,K], scales uint16 fp16-bits [N])."""
    W = _bits(W)
    if W.ndim != 2:
        raise ValueError("W must be [N,K]")
    N, K = W.shape
    codes = np.zeros((N, K), np.uint8)
    scales = np.zeros(N, np.uint16)
    st = lib().fp6o_quantize(_ptr(W), N, K, _ptr(codes), _ptr(scales))
    if st != 0:
        raise ValueError("oracle: quantize failed (status %d)" % st)
    return codes, scales


def split42(codes):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    hi4 = np.zeros_like(codes)
    lo2 = np.zeros_like(codes)
    lib().fp6o_split42(_ptr(codes), codes.size, _ptr(hi4), _ptr(lo2))
    return hi4, lo2


def join42(hi4, lo2):
    hi4 = np.ascontiguousarray(hi4, dtype=np.uint8)
    lo2 = np.ascontiguousarray(lo2, dtype=np.uint8)
    codes = np.zeros_like(hi4)
    lib().fp6o_join42(_ptr(hi4), _ptr(lo2), hi4.size, _ptr(codes))
    return codes


def dequantize(codes, scales) -> np.ndarray:
    """-> W_hat as uint16 fp16 bit patterns [N,K]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales).reshape(-1)
    N, K = codes.shape
    assert scales.size == N
    out = np.zeros((N, K), np.uint16)
    lib().fp6o_dequantize(_ptr(codes), _ptr(scales), N, K, _ptr(out))
    return out


def linear(X, codes, scales) -> np.ndarray:
    """X fp16 [M,K]; codes [N,K]; scales fp16 [N] -> Y float64 [M,N]."""
    X = _bits(X)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales).reshape(-1)
    M, K = X.shape
    N, K2 = codes.shape
    assert K == K2 and scales.size == N
    Y = np.zeros((M, N), np.float64)
    lib().fp6o_linear(_ptr(X), M, _ptr(codes), _ptr(scales), N, K, _ptr(Y))
    return Y


# ---- bf16 activations (Section 2: FP16 or BF16 around the FP6 weights)

def bf16_to_double(bits: int) -> float:
    return float(lib().fp6o_bf16_to_double(int(bits) & 0xFFFF))


def double_to_bf16(x: float) -> int:
    """Round to nearest, ties to even; finite x inside the bf16 range."""
    return int(lib().fp6o_double_to_bf16(float(x)))


def linear_bf16(X, codes, scales) -> np.ndarray:
    """X bf16 bit patterns (uint16) [M,K]; codes [N,K]; scales fp16 [N] -> Y float64 [M,N]."""
    X = np.ascontiguousarray(X, dtype=np.uint16)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales).reshape(-1)
    M, K = X.shape
    N, K2 = codes.shape
    assert K == K2 and scales.size == N
    Y = np.zeros((M, N), np.float64)
    lib().fp6o_linear_bf16(_ptr(X), M, _ptr(codes), _ptr(scales), N, K, _ptr(Y))
    return Y


# ---- fine-grained (block-k) scales: Section 3 "FGQ", Appendix A "block-k quantization"

def quantize_fgq(W, block: int):
    """W fp16 [N,K] -> (codes uint8 [N,K], scales uint16 fp16-bits [N, K/block])."""
    W = _bits(W)
    if W.ndim != 2:
        raise ValueError("W must be [N,K]")
    N, K = W.shape
    if block <= 0 or K % block:
        raise ValueError("block must divide K")
    codes = np.zeros((N, K), np.uint8)
    scales = np.zeros((N, K // block), np.uint16)
    st = lib().fp6o_quantize_fgq(_ptr(W), N, K, block, _ptr(codes), _ptr(scales))
    if st != 0:
        raise ValueError("oracle: quantize_fgq failed (status %d)" % st)
    return codes, scales


def dequantize_fgq(codes, scales, block: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales)
    N, K = codes.shape
    assert scales.shape == (N, K // block)
    out = np.zeros((N, K), np.uint16)
    lib().fp6o_dequantize_fgq(_ptr(codes), _ptr(scales), N, K, block, _ptr(out))
    return out


def linear_fgq(X, codes, scales, block: int) -> np.ndarray:
    """X fp16 [M,K]; codes [N,K]; scales fp16 [N,K/block] -> Y float64 [M,N]."""
    X = _bits(X)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales)
    M, K = X.shape
    N, K2 = codes.shape
    assert K == K2 and scales.shape == (N, K // block)
    Y = np.zeros((M, N), np.float64)
    lib().fp6o_linear_fgq(_ptr(X), M, _ptr(codes), _ptr(scales), N, K, block, _ptr(Y))
    return Y


# ---- FP5 E3M1, "4+1" (Section 4 last sentence; Section 6)

def e3m1_value(code: int) -> float:
    return float(lib().fp5o_e3m1_value(int(code)))


def bias_shift_bits5(code: int) -> int:
    return int(lib().fp5o_bias_shift_bits(int(code)))


def quantize5(W):
    """W fp16 [N,K] -> (codes uint8 [N,K] in 0..31, scales uint16 fp16-bits [N]); S = max|w| / 24."""
    W = _bits(W)
    if W.ndim != 2:
        raise ValueError("W must be [N,K]")
    N, K = W.shape
    codes = np.zeros((N, K), np.uint8)
    scales = np.zeros(N, np.uint16)
    st = lib().fp5o_quantize(_ptr(W), N, K, _ptr(codes), _ptr(scales))
    if st != 0:
        raise ValueError("oracle: quantize5 failed (status %d)" % st)
    return codes, scales


def split41(codes):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    hi4 = np.zeros_like(codes)
    lo1 = np.zeros_like(codes)
    lib().fp5o_split41(_ptr(codes), codes.size, _ptr(hi4), _ptr(lo1))
    return hi4, lo1


def dequantize5(codes, scales) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales).reshape(-1)
    N, K = codes.shape
    assert scales.size == N
    out = np.zeros((N, K), np.uint16)
    lib().fp5o_dequantize(_ptr(codes), _ptr(scales), N, K, _ptr(out))
    return out


def linear5(X, codes, scales) -> np.ndarray:
    X = _bits(X)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = _bits(scales).reshape(-1)
    M, K = X.shape
    N, K2 = codes.shape
    assert K == K2 and scales.size == N
    Y = np.zeros((M, N), np.float64)
    lib().fp5o_linear(_ptr(X), M, _ptr(codes), _ptr(scales), N, K, _ptr(Y))
    return Y
