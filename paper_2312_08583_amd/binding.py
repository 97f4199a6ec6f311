"""Thin ctypes binding of libfp6_linear.so (the C ABI in include/fp6_linear.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch is
used for device memory and for the current stream, nothing else.  There is no CPU
fallback: if the library cannot be loaded, or a tensor is not on the GPU, the call
raises.
"""
import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FP6_LINEAR_LIB", os.path.join(_HERE, "libfp6_linear.so"))   # override: tuning builds

FP6_TILE = 64
FP6_OK = 0
FP6_VARIANT_AUTO, FP6_VARIANT_DECODE, FP6_VARIANT_GEMM = 0, 1, 2
FP6_WORKSPACE_ZERO_BYTES = 4259840


# tuning hints carried in the upper bits of `variant` (same macros as the header)
def FP6_HINT_WAVES(w: int) -> int:
    return int(w) << 8


def FP6_HINT_DEPTH(d: int) -> int:
    return int(d) << 12


def FP6_HINT_BLOCK_M(b: int) -> int:
    return (int(b) // 16) << 16


def FP6_HINT_MEET(x: int) -> int:
    return int(x) << 20


def FP6_HINT_DEQUANT(x: int) -> int:
    return int(x) << 22


def FP6_HINT_HALF(x: int) -> int:
    return int(x) << 24


def FP6_HINT_WIDTH(b: int) -> int:
    return int(b) << 26


EXPORTS = ["fp6_layout_version", "fp6_status_string", "fp6_packed_sizes", "fp6_quantize_pack",
           "fp6_unpack_codes", "fp6_dequantize", "fp6_linear_workspace_bytes", "fp6_linear",
           "fp6_linear_variant_workspace_bytes", "fp6_linear_variant", "fp6_quantize_pack_fgq",
           "fp6_dequantize_fgq", "fp6_linear_fgq_workspace_bytes", "fp6_linear_fgq", "fp5_packed_sizes",
           "fp5_quantize_pack", "fp5_unpack_codes", "fp5_dequantize", "fp5_linear_workspace_bytes", "fp5_linear",
           "fp6_quantize_pack_v2", "fp6_unpack_codes_v2", "fp6_dequantize_v2", "fp6_linear_v2_workspace_bytes",
           "fp6_linear_v2", "fp6_linear_v2_bf16", "fp6_probe_read", "fp6_probe_mfma"]

_LIB = None


class Fp6Error(RuntimeError):
    pass


def lib() -> ctypes.CDLL:
    """Load the built library (building it first only if no built library exists)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(LIB_PATH)
    i64, p, sz, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    L.fp6_layout_version.restype = ci
    L.fp6_layout_version.argtypes = []
    L.fp6_status_string.restype = ctypes.c_char_p
    L.fp6_status_string.argtypes = [ci]
    L.fp6_packed_sizes.restype = ci
    L.fp6_packed_sizes.argtypes = [i64, i64, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.fp6_quantize_pack.restype = ci
    L.fp6_quantize_pack.argtypes = [p, i64, i64, p, p, p, p]
    L.fp6_unpack_codes.restype = ci
    L.fp6_unpack_codes.argtypes = [p, p, i64, i64, p, p]
    L.fp6_dequantize.restype = ci
    L.fp6_dequantize.argtypes = [p, p, p, i64, i64, p, p]
    L.fp6_linear_workspace_bytes.restype = sz
    L.fp6_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.fp6_linear.restype = ci
    L.fp6_linear.argtypes = [p, i64, p, p, p, i64, i64, p, p, sz, p]
    L.fp6_linear_variant_workspace_bytes.restype = sz
    L.fp6_linear_variant_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    L.fp6_linear_variant.restype = ci
    L.fp6_linear_variant.argtypes = [p, i64, p, p, p, i64, i64, p, p, sz, p, ci, ci]
    L.fp6_quantize_pack_fgq.restype = ci
    L.fp6_quantize_pack_fgq.argtypes = [p, i64, i64, i64, p, p, p, p]
    L.fp6_dequantize_fgq.restype = ci
    L.fp6_dequantize_fgq.argtypes = [p, p, p, i64, i64, i64, p, p]
    L.fp6_linear_fgq_workspace_bytes.restype = sz
    L.fp6_linear_fgq_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, ci]
    L.fp6_linear_fgq.restype = ci
    L.fp6_linear_fgq.argtypes = [p, i64, p, p, p, i64, i64, i64, p, p, sz, p, ci, ci]
    L.fp5_packed_sizes.restype = ci
    L.fp5_packed_sizes.argtypes = [i64, i64, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.fp5_quantize_pack.restype = ci
    L.fp5_quantize_pack.argtypes = [p, i64, i64, p, p, p, p]
    L.fp5_unpack_codes.restype = ci
    L.fp5_unpack_codes.argtypes = [p, p, i64, i64, p, p]
    L.fp5_dequantize.restype = ci
    L.fp5_dequantize.argtypes = [p, p, p, i64, i64, p, p]
    L.fp5_linear_workspace_bytes.restype = sz
    L.fp5_linear_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    L.fp5_linear.restype = ci
    L.fp5_linear.argtypes = [p, i64, p, p, p, i64, i64, p, p, sz, p, ci, ci]
    L.fp6_quantize_pack_v2.restype = ci
    L.fp6_quantize_pack_v2.argtypes = [p, i64, i64, p, p, p, p]
    L.fp6_unpack_codes_v2.restype = ci
    L.fp6_unpack_codes_v2.argtypes = [p, p, i64, i64, p, p]
    L.fp6_dequantize_v2.restype = ci
    L.fp6_dequantize_v2.argtypes = [p, p, p, i64, i64, p, p]
    L.fp6_linear_v2_workspace_bytes.restype = sz
    L.fp6_linear_v2_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    L.fp6_linear_v2.restype = ci
    L.fp6_linear_v2.argtypes = [p, i64, p, p, p, i64, i64, p, p, sz, p, ci, ci]
    L.fp6_linear_v2_bf16.restype = ci
    L.fp6_linear_v2_bf16.argtypes = [p, i64, p, p, p, i64, i64, p, p, sz, p, ci, ci]
    L.fp6_probe_read.restype = ci
    L.fp6_probe_read.argtypes = [p, sz, ci, p, sz, p]
    L.fp6_probe_mfma.restype = ci
    L.fp6_probe_mfma.argtypes = [ci, ci, ci, ci, p, sz, p]
    _LIB = L
    return L


def fp6_status_string(status: int) -> str:
    return lib().fp6_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != FP6_OK:
        raise Fp6Error("%s failed: %s (status %d)" % (what, fp6_status_string(status), status))


def _dev(t: torch.Tensor, dtype, what: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise Fp6Error("%s must be a GPU tensor (this library has no CPU path)" % what)
    if t.dtype != dtype or not t.is_contiguous():
        raise Fp6Error("%s must be contiguous %s" % (what, dtype))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def fp6_layout_version() -> int:
    return int(lib().fp6_layout_version())


def fp6_packed_sizes(N: int, K: int) -> Tuple[int, int, int]:
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().fp6_packed_sizes(N, K, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fp6_packed_sizes")
    return a.value, b.value, c.value


def fp6_quantize_pack(W: torch.Tensor):
    """W fp16 [N,K] on the GPU -> (hi_plane uint8 [N*K/2], lo_plane uint8 [N*K/4], scales fp16 [N])."""
    wp = _dev(W, torch.float16, "W")
    N, K = W.shape
    hb, lb, _ = fp6_packed_sizes(N, K)
    hi = torch.empty(hb, dtype=torch.uint8, device=W.device)
    lo = torch.empty(lb, dtype=torch.uint8, device=W.device)
    scales = torch.empty(N, dtype=torch.float16, device=W.device)
    _check(lib().fp6_quantize_pack(wp, N, K, hi.data_ptr(), lo.data_ptr(), scales.data_ptr(), _stream()),
           "fp6_quantize_pack")
    return hi, lo, scales


def fp6_unpack_codes(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int) -> torch.Tensor:
    codes = torch.empty((N, K), dtype=torch.uint8, device=hi.device)
    _check(lib().fp6_unpack_codes(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"), N, K,
                                  codes.data_ptr(), _stream()), "fp6_unpack_codes")
    return codes


def fp6_dequantize(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.float16, device=hi.device)
    _check(lib().fp6_dequantize(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                _dev(scales, torch.float16, "scales"), N, K, out.data_ptr(), _stream()),
           "fp6_dequantize")
    return out


def fp6_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().fp6_linear_workspace_bytes(M, N, K))


def fp6_linear_variant_workspace_bytes(M: int, N: int, K: int, variant: int, split_k: int) -> int:
    return int(lib().fp6_linear_variant_workspace_bytes(M, N, K, variant, split_k))


def new_workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    """Zero-filled workspace (the counters at its start must be zero before first use)."""
    if nbytes == 0:
        return None
    return torch.zeros(nbytes, dtype=torch.uint8, device=device)


def fp6_linear_variant(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                       variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    xp = _dev(X, torch.float16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [M,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    need = fp6_linear_variant_workspace_bytes(M, N, K, variant, split_k)
    if workspace is None:
        workspace = new_workspace(need, X.device)
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp6_linear_variant(xp, M, _dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                    _dev(scales, torch.float16, "scales"), N, K,
                                    _dev(out, torch.float16, "Y"), wp, wb, _stream(), variant, split_k),
           "fp6_linear_variant")
    return out


def fp6_linear(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M,N] = X[M,K] x dequant(planes)^T with the row scales applied after the accumulation."""
    xp = _dev(X, torch.float16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [M,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = new_workspace(fp6_linear_workspace_bytes(M, N, K), X.device)
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp6_linear(xp, M, _dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                            _dev(scales, torch.float16, "scales"), N, K, _dev(out, torch.float16, "Y"),
                            wp, wb, _stream()), "fp6_linear")
    return out


# ---- fine-grained (block-k) scales

def fp6_quantize_pack_fgq(W: torch.Tensor, block: int):
    """W fp16 [N,K] -> (hi_plane, lo_plane, scales fp16 [K/block, N]): one scale per `block` elements of a row."""
    wp = _dev(W, torch.float16, "W")
    N, K = W.shape
    hb, lb, _ = fp6_packed_sizes(N, K)
    if block <= 0 or K % block:
        raise Fp6Error("block must divide K")
    hi = torch.empty(hb, dtype=torch.uint8, device=W.device)
    lo = torch.empty(lb, dtype=torch.uint8, device=W.device)
    scales = torch.empty((K // block, N), dtype=torch.float16, device=W.device)
    _check(lib().fp6_quantize_pack_fgq(wp, N, K, block, hi.data_ptr(), lo.data_ptr(), scales.data_ptr(), _stream()),
           "fp6_quantize_pack_fgq")
    return hi, lo, scales


def fp6_dequantize_fgq(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                       block: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.float16, device=hi.device)
    _check(lib().fp6_dequantize_fgq(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                    _dev(scales, torch.float16, "scales"), N, K, block, out.data_ptr(), _stream()),
           "fp6_dequantize_fgq")
    return out


def fp6_linear_fgq_workspace_bytes(M: int, N: int, K: int, block: int, variant: int = FP6_VARIANT_AUTO,
                                   split_k: int = 0) -> int:
    return int(lib().fp6_linear_fgq_workspace_bytes(M, N, K, block, variant, split_k))


def fp6_linear_fgq(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                   block: int, variant: int = FP6_VARIANT_AUTO, split_k: int = 0,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M,N] with block scales applied to each block's product sum before the accumulation."""
    xp = _dev(X, torch.float16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [M,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = new_workspace(fp6_linear_fgq_workspace_bytes(M, N, K, block, variant, split_k), X.device)
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp6_linear_fgq(xp, M, _dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                _dev(scales, torch.float16, "scales"), N, K, block, _dev(out, torch.float16, "Y"),
                                wp, wb, _stream(), variant, split_k), "fp6_linear_fgq")
    return out


# ---- FP5 E3M1 ("4+1")

def fp5_packed_sizes(N: int, K: int) -> Tuple[int, int, int]:
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().fp5_packed_sizes(N, K, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fp5_packed_sizes")
    return a.value, b.value, c.value


def fp5_quantize_pack(W: torch.Tensor):
    """W fp16 [N,K] -> (hi_plane uint8 [N*K/2], lo_plane uint8 [N*K/8], scales fp16 [N])."""
    wp = _dev(W, torch.float16, "W")
    N, K = W.shape
    hb, lb, _ = fp5_packed_sizes(N, K)
    hi = torch.empty(hb, dtype=torch.uint8, device=W.device)
    lo = torch.empty(lb, dtype=torch.uint8, device=W.device)
    scales = torch.empty(N, dtype=torch.float16, device=W.device)
    _check(lib().fp5_quantize_pack(wp, N, K, hi.data_ptr(), lo.data_ptr(), scales.data_ptr(), _stream()),
           "fp5_quantize_pack")
    return hi, lo, scales


def fp5_unpack_codes(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int) -> torch.Tensor:
    codes = torch.empty((N, K), dtype=torch.uint8, device=hi.device)
    _check(lib().fp5_unpack_codes(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"), N, K,
                                  codes.data_ptr(), _stream()), "fp5_unpack_codes")
    return codes


def fp5_dequantize(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.float16, device=hi.device)
    _check(lib().fp5_dequantize(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                _dev(scales, torch.float16, "scales"), N, K, out.data_ptr(), _stream()),
           "fp5_dequantize")
    return out


def fp5_linear_workspace_bytes(M: int, N: int, K: int, variant: int = FP6_VARIANT_AUTO, split_k: int = 0) -> int:
    return int(lib().fp5_linear_workspace_bytes(M, N, K, variant, split_k))


def fp5_linear(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
               variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    xp = _dev(X, torch.float16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [M,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = new_workspace(fp5_linear_workspace_bytes(M, N, K, variant, split_k), X.device)
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp5_linear(xp, M, _dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                            _dev(scales, torch.float16, "scales"), N, K, _dev(out, torch.float16, "Y"),
                            wp, wb, _stream(), variant, split_k), "fp5_linear")
    return out


# ---- FP6 in plane layout 2 (hardware conversion)

def fp6_quantize_pack_v2(W: torch.Tensor):
    wp = _dev(W, torch.float16, "W")
    N, K = W.shape
    hb, lb, _ = fp6_packed_sizes(N, K)
    hi = torch.empty(hb, dtype=torch.uint8, device=W.device)
    lo = torch.empty(lb, dtype=torch.uint8, device=W.device)
    scales = torch.empty(N, dtype=torch.float16, device=W.device)
    _check(lib().fp6_quantize_pack_v2(wp, N, K, hi.data_ptr(), lo.data_ptr(), scales.data_ptr(), _stream()),
           "fp6_quantize_pack_v2")
    return hi, lo, scales


def fp6_unpack_codes_v2(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int) -> torch.Tensor:
    codes = torch.empty((N, K), dtype=torch.uint8, device=hi.device)
    _check(lib().fp6_unpack_codes_v2(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"), N, K,
                                     codes.data_ptr(), _stream()), "fp6_unpack_codes_v2")
    return codes


def fp6_dequantize_v2(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.float16, device=hi.device)
    _check(lib().fp6_dequantize_v2(_dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                   _dev(scales, torch.float16, "scales"), N, K, out.data_ptr(), _stream()),
           "fp6_dequantize_v2")
    return out


def fp6_linear_v2_workspace_bytes(M: int, N: int, K: int, variant: int = FP6_VARIANT_AUTO, split_k: int = 0) -> int:
    return int(lib().fp6_linear_v2_workspace_bytes(M, N, K, variant, split_k))


def fp6_linear_v2(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                  variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    xp = _dev(X, torch.float16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [M,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    if workspace is None:
        workspace = new_workspace(fp6_linear_v2_workspace_bytes(M, N, K, variant, split_k), X.device)
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp6_linear_v2(xp, M, _dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                               _dev(scales, torch.float16, "scales"), N, K, _dev(out, torch.float16, "Y"),
                               wp, wb, _stream(), variant, split_k), "fp6_linear_v2")
    return out


def fp6_probe_read(buf: torch.Tensor, workgroups: int, sink: torch.Tensor) -> None:
    """One launch of the plain read kernel over all bytes of `buf` (a contiguous device tensor)."""
    if not (buf.is_cuda and buf.is_contiguous() and sink.is_cuda and sink.is_contiguous()):
        raise Fp6Error("buf and sink must be contiguous device tensors")
    _check(lib().fp6_probe_read(buf.data_ptr(), buf.numel() * buf.element_size(), workgroups, sink.data_ptr(),
                                sink.numel() * sink.element_size(), _stream()), "fp6_probe_read")


def fp6_probe_mfma(workgroups: int, iters: int, random_operands: bool, sink: torch.Tensor, wide: bool = False) -> int:
    """One launch of the MFMA-only kernel; returns the flop count of the launch."""
    if not (sink.is_cuda and sink.is_contiguous()):
        raise Fp6Error("sink must be a contiguous device tensor")
    _check(lib().fp6_probe_mfma(workgroups, iters, int(bool(random_operands)), int(bool(wide)), sink.data_ptr(),
                                sink.numel() * sink.element_size(), _stream()), "fp6_probe_mfma")
    return workgroups * 4 * 8 * iters * 16384 * (2 if wide else 1)


def fp6_linear_v2_bf16(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                       variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Layout-2 planes against bf16 activations; returns bf16."""
    xp = _dev(X, torch.bfloat16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K:
        raise Fp6Error("X must be [M,K]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    if workspace is None:
        workspace = new_workspace(fp6_linear_v2_workspace_bytes(M, N, K, variant, split_k), X.device)
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp6_linear_v2_bf16(xp, M, _dev(hi, torch.uint8, "hi_plane"), _dev(lo, torch.uint8, "lo_plane"),
                                    _dev(scales, torch.float16, "scales"), N, K, _dev(out, torch.bfloat16, "Y"),
                                    wp, wb, _stream(), variant, split_k), "fp6_linear_v2_bf16")
    return out
