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


def FP6_HINT_KWAYS(x: int) -> int:
    return int(int(x) == 2) << 30


EXPORTS = ["fp6_layout_version", "fp6_status_string", "fp6_packed_sizes", "fp6_quantize_pack",
           "fp6_unpack_codes", "fp6_dequantize", "fp6_linear_workspace_bytes", "fp6_linear",
           "fp6_linear_variant_workspace_bytes", "fp6_linear_variant", "fp6_quantize_pack_fgq",
           "fp6_dequantize_fgq", "fp6_linear_fgq_workspace_bytes", "fp6_linear_fgq", "fp5_packed_sizes",
           "fp5_quantize_pack", "fp5_unpack_codes", "fp5_dequantize", "fp5_linear_workspace_bytes", "fp5_linear",
           "fp6_quantize_pack_v2", "fp6_unpack_codes_v2", "fp6_dequantize_v2", "fp6_linear_v2_workspace_bytes",
           "fp6_linear_v2", "fp6_linear_v2_bf16", "fp6_probe_read", "fp6_probe_mfma", "fp6_linear_plan", "fp6_linear_static", "fp6_linear_group",
           "fp6_linear_group_workspace_bytes"]

FP6_FORMAT_E3M2, FP6_FORMAT_E3M1, FP6_FORMAT_E3M2_V2, FP6_FORMAT_E3M2_V2_BF16 = 6, 5, 7, 8


FP6_GROUP_MAX = 4


class LinearProblem(ctypes.Structure):
    """fp6_linear_problem of the header."""
    _fields_ = [("X", ctypes.c_void_p), ("hi_plane", ctypes.c_void_p), ("lo_plane", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("Y", ctypes.c_void_p)]


class PlanInfo(ctypes.Structure):
    """fp6_plan_info of the header."""
    _fields_ = [("variant", ctypes.c_int), ("split_k", ctypes.c_int), ("block_m", ctypes.c_int), ("width", ctypes.c_int),
                ("waves", ctypes.c_int), ("depth", ctypes.c_int), ("half_tiles", ctypes.c_int), ("meeting", ctypes.c_int),
                ("workgroups", ctypes.c_int64), ("workspace_bytes", ctypes.c_size_t)]

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
    L.fp6_linear_static.restype = ci
    L.fp6_linear_static.argtypes = [p, i64, p, p, p, i64, i64, p, p]
    L.fp6_linear_group_workspace_bytes.restype = sz
    L.fp6_linear_group_workspace_bytes.argtypes = [i64, ctypes.POINTER(LinearProblem), ci]
    L.fp6_linear_group.restype = ci
    L.fp6_linear_group.argtypes = [i64, ctypes.POINTER(LinearProblem), ci, p, sz, p]
    L.fp6_linear_plan.restype = ci
    L.fp6_linear_plan.argtypes = [ci, i64, i64, i64, i64, ci, ci, ctypes.POINTER(PlanInfo)]
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


def _sized(t: torch.Tensor, dtype, what: str, numel: int) -> int:
    """Device pointer of `t` after checking that it holds exactly `numel` elements: the C ABI sees pointers
    only, so this is the one place where a buffer that is too small for (N, K) can be stopped."""
    ptr = _dev(t, dtype, what)
    if t.numel() != numel:
        raise Fp6Error("%s holds %d elements, the shape needs %d" % (what, t.numel(), numel))
    return ptr


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _shape_ok(N: int, K: int) -> None:
    if N <= 0 or K <= 0 or N % FP6_TILE or K % FP6_TILE:
        raise Fp6Error("N and K must be positive multiples of %d" % FP6_TILE)


def _planes(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int, lo_div: int = 4) -> Tuple[int, int]:
    """Pointers of the two planes, sized for [N, K]: N*K/2 bytes and N*K/lo_div bytes."""
    _shape_ok(N, K)
    return _sized(hi, torch.uint8, "hi_plane", N * K // 2), _sized(lo, torch.uint8, "lo_plane", N * K // lo_div)


def fp6_layout_version() -> int:
    return int(lib().fp6_layout_version())


def fp6_packed_sizes(N: int, K: int) -> Tuple[int, int, int]:
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().fp6_packed_sizes(N, K, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fp6_packed_sizes")
    return a.value, b.value, c.value


def fp5_packed_sizes(N: int, K: int) -> Tuple[int, int, int]:
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().fp5_packed_sizes(N, K, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "fp5_packed_sizes")
    return a.value, b.value, c.value


def fp6_linear_plan(M: int, N: int, K: int, format: int = FP6_FORMAT_E3M2, block: int = 0,
                    variant: int = FP6_VARIANT_AUTO, split_k: int = 0) -> dict:
    """What the hot-path call for this shape would launch (host-only query; needs no GPU)."""
    info = PlanInfo()
    _check(lib().fp6_linear_plan(format, M, N, K, block, variant, split_k, ctypes.byref(info)), "fp6_linear_plan")
    return {name: int(getattr(info, name)) for name, _ in PlanInfo._fields_}


def plan_text(plan: dict) -> str:
    """One-line summary of a plan for benchmark rows."""
    fam = "decode" if plan["variant"] == FP6_VARIANT_DECODE else "gemm"
    meet = ("", " counter", " pairwise")[plan["meeting"]]
    if fam == "decode":
        return "decode%s rows%d split%d%s wg%d" % (" half" if plan["half_tiles"] else "", plan["block_m"], plan["split_k"],
                                                   meet, plan["workgroups"])
    kways = " k%d" % (plan["waves"] // plan["width"]) if plan["waves"] > plan["width"] else ""
    return "gemm %dx%d%s split%d%s wg%d" % (plan["block_m"], 64 * plan["width"], kways, plan["split_k"], meet,
                                            plan["workgroups"])


def new_workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    """Zero-filled workspace (the counters at its start must be zero before first use)."""
    if nbytes == 0:
        return None
    return torch.zeros(nbytes, dtype=torch.uint8, device=device)


# ---- offline step and test utilities: one marshalling routine per kind of call

def _quantize_pack(name: str, W: torch.Tensor, sizes, block: int = 0):
    wp = _dev(W, torch.float16, "W")
    if W.dim() != 2:
        raise Fp6Error("W must be [N,K]")
    N, K = W.shape
    hb, lb, _ = sizes(N, K)
    if block and (block <= 0 or K % block):
        raise Fp6Error("block must divide K")
    hi = torch.empty(hb, dtype=torch.uint8, device=W.device)
    lo = torch.empty(lb, dtype=torch.uint8, device=W.device)
    scales = torch.empty((K // block, N) if block else (N,), dtype=torch.float16, device=W.device)
    fn = getattr(lib(), name)
    args = (wp, N, K) + ((block,) if block else ()) + (hi.data_ptr(), lo.data_ptr(), scales.data_ptr(), _stream())
    _check(fn(*args), name)
    return hi, lo, scales


def _unpack_codes(name: str, hi, lo, N: int, K: int, lo_div: int) -> torch.Tensor:
    hp, lp = _planes(hi, lo, N, K, lo_div)
    codes = torch.empty((N, K), dtype=torch.uint8, device=hi.device)
    _check(getattr(lib(), name)(hp, lp, N, K, codes.data_ptr(), _stream()), name)
    return codes


def _dequantize(name: str, hi, lo, scales, N: int, K: int, lo_div: int, block: int = 0) -> torch.Tensor:
    hp, lp = _planes(hi, lo, N, K, lo_div)
    if block and (block <= 0 or K % block):
        raise Fp6Error("block must divide K")
    sp = _sized(scales, torch.float16, "scales", N * (K // block if block else 1))
    out = torch.empty((N, K), dtype=torch.float16, device=hi.device)
    args = (hp, lp, sp, N, K) + ((block,) if block else ()) + (out.data_ptr(), _stream())
    _check(getattr(lib(), name)(*args), name)
    return out


def _linear(name: str, need, X, hi, lo, scales, N: int, K: int, out, workspace, tail=(), block: int = 0,
            lo_div: int = 4, dtype=torch.float16) -> torch.Tensor:
    """Marshal one hot-path call: every buffer is checked against the sizes that (M, N, K) imply."""
    if not isinstance(X, torch.Tensor) or X.dim() != 2 or X.shape[1] != K or X.shape[0] < 1:
        raise Fp6Error("X must be [M,K] with M >= 1")
    xp = _dev(X, dtype, "X")
    M = X.shape[0]
    hp, lp = _planes(hi, lo, N, K, lo_div)
    if block and (block <= 0 or K % block):
        raise Fp6Error("block must divide K")
    sp = _sized(scales, torch.float16, "scales", N * (K // block if block else 1))
    if out is None:
        out = torch.empty((M, N), dtype=dtype, device=X.device)
    elif tuple(out.shape) != (M, N):
        raise Fp6Error("Y must be [M,N] = [%d,%d], got %s" % (M, N, tuple(out.shape)))
    yp = _dev(out, dtype, "Y")
    if workspace is None:
        workspace = new_workspace(int(need(M)), X.device)      # `need`: workspace bytes as a function of M
    elif not (isinstance(workspace, torch.Tensor) and workspace.is_cuda and workspace.is_contiguous()
              and workspace.dtype == torch.uint8):
        raise Fp6Error("workspace must be a contiguous uint8 GPU tensor")
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    args = (xp, M, hp, lp, sp, N, K) + ((block,) if block else ()) + (yp, wp, wb, _stream()) + tuple(tail)
    _check(getattr(lib(), name)(*args), name)
    return out


def fp6_quantize_pack(W: torch.Tensor):
    """W fp16 [N,K] on the GPU -> (hi_plane uint8 [N*K/2], lo_plane uint8 [N*K/4], scales fp16 [N])."""
    return _quantize_pack("fp6_quantize_pack", W, fp6_packed_sizes)


def fp6_unpack_codes(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int) -> torch.Tensor:
    return _unpack_codes("fp6_unpack_codes", hi, lo, N, K, 4)


def fp6_dequantize(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int) -> torch.Tensor:
    return _dequantize("fp6_dequantize", hi, lo, scales, N, K, 4)


def fp6_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().fp6_linear_workspace_bytes(M, N, K))


def fp6_linear_variant_workspace_bytes(M: int, N: int, K: int, variant: int, split_k: int) -> int:
    return int(lib().fp6_linear_variant_workspace_bytes(M, N, K, variant, split_k))


def fp6_linear_variant(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                       variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    need = lambda M: fp6_linear_variant_workspace_bytes(M, N, K, variant, split_k)
    return _linear("fp6_linear_variant", need, X, hi, lo, scales, N, K, out, workspace, (variant, split_k))


def fp6_linear(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
               out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M,N] = X[M,K] x dequant(planes)^T with the row scales applied after the accumulation."""
    need = lambda M: fp6_linear_workspace_bytes(M, N, K)
    return _linear("fp6_linear", need, X, hi, lo, scales, N, K, out, workspace)


FP6_STATIC_SCRATCH_BYTES = 67108864
FP6_ERR_SCRATCH = -7


def fp6_linear_static(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """fp6_linear on the library's built-in scratch: no workspace argument, nothing allocated by the call
    (pass `out`; without it this wrapper, not the library, allocates Y)."""
    if not isinstance(X, torch.Tensor) or X.dim() != 2 or X.shape[1] != K or X.shape[0] < 1:
        raise Fp6Error("X must be [M,K] with M >= 1")
    xp = _dev(X, torch.float16, "X")
    M = X.shape[0]
    hp, lp = _planes(hi, lo, N, K)
    sp = _sized(scales, torch.float16, "scales", N)
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    elif tuple(out.shape) != (M, N):
        raise Fp6Error("Y must be [M,N] = [%d,%d], got %s" % (M, N, tuple(out.shape)))
    _check(lib().fp6_linear_static(xp, M, hp, lp, sp, N, K, _dev(out, torch.float16, "Y"), _stream()), "fp6_linear_static")
    return out


def _group_array(layers, M: Optional[int] = None, outs=None):
    """(X, hi, lo, scales, N, K) per layer -> checked ctypes array of fp6_linear_problem, M, list of Y tensors."""
    if not 1 <= len(layers) <= FP6_GROUP_MAX:
        raise Fp6Error("a group holds 1 to %d layers" % FP6_GROUP_MAX)
    arr = (LinearProblem * len(layers))()
    ys = []
    for i, (X, hi, lo, scales, N, K) in enumerate(layers):
        if not isinstance(X, torch.Tensor) or X.dim() != 2 or X.shape[1] != K or X.shape[0] < 1:
            raise Fp6Error("X must be [M,K] with M >= 1")
        if M is None:
            M = X.shape[0]
        if X.shape[0] != M:
            raise Fp6Error("the layers of a group share M")
        hp, lp = _planes(hi, lo, N, K)
        Y = None if outs is None else outs[i]
        if Y is None:
            Y = torch.empty((M, N), dtype=torch.float16, device=X.device)
        elif tuple(Y.shape) != (M, N):
            raise Fp6Error("Y must be [M,N] = [%d,%d], got %s" % (M, N, tuple(Y.shape)))
        arr[i] = LinearProblem(_dev(X, torch.float16, "X"), hp, lp, _sized(scales, torch.float16, "scales", N), N, K,
                               _dev(Y, torch.float16, "Y"))
        ys.append(Y)
    return arr, M, ys


def fp6_linear_group_workspace_bytes(M: int, shapes) -> int:
    """Workspace for a group of layers given as (N, K) pairs (the pointers do not enter the size)."""
    arr = (LinearProblem * len(shapes))()
    for i, (N, K) in enumerate(shapes):
        arr[i] = LinearProblem(16, 16, 16, 16, N, K, 16)        # aligned non-NULL placeholders, never dereferenced
    return int(lib().fp6_linear_group_workspace_bytes(M, arr, len(shapes)))


def fp6_linear_group(layers, outs=None, workspace: Optional[torch.Tensor] = None):
    """Independent layers [(X, hi, lo, scales, N, K), ...] on activations of one height M in one call
    (one launch for M <= 16 and a common K).  Returns the list of Y tensors."""
    arr, M, ys = _group_array(layers, outs=outs)
    need = int(lib().fp6_linear_group_workspace_bytes(M, arr, len(layers)))
    if workspace is None:
        workspace = new_workspace(need, ys[0].device)
    elif not (isinstance(workspace, torch.Tensor) and workspace.is_cuda and workspace.is_contiguous()
              and workspace.dtype == torch.uint8):
        raise Fp6Error("workspace must be a contiguous uint8 GPU tensor")
    wp = workspace.data_ptr() if workspace is not None else None
    wb = workspace.numel() if workspace is not None else 0
    _check(lib().fp6_linear_group(M, arr, len(layers), wp, wb, _stream()), "fp6_linear_group")
    return ys


# ---- fine-grained (block-k) scales

def fp6_quantize_pack_fgq(W: torch.Tensor, block: int):
    """W fp16 [N,K] -> (hi_plane, lo_plane, scales fp16 [K/block, N]): one scale per `block` elements of a row."""
    if block <= 0:
        raise Fp6Error("block must divide K")
    return _quantize_pack("fp6_quantize_pack_fgq", W, fp6_packed_sizes, block)


def fp6_dequantize_fgq(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                       block: int) -> torch.Tensor:
    if block <= 0:
        raise Fp6Error("block must divide K")
    return _dequantize("fp6_dequantize_fgq", hi, lo, scales, N, K, 4, block)


def fp6_linear_fgq_workspace_bytes(M: int, N: int, K: int, block: int, variant: int = FP6_VARIANT_AUTO,
                                   split_k: int = 0) -> int:
    return int(lib().fp6_linear_fgq_workspace_bytes(M, N, K, block, variant, split_k))


def fp6_linear_fgq(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                   block: int, variant: int = FP6_VARIANT_AUTO, split_k: int = 0,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y[M,N] with block scales applied to each block's product sum before the accumulation."""
    if block <= 0:
        raise Fp6Error("block must divide K")
    need = lambda M: fp6_linear_fgq_workspace_bytes(M, N, K, block, variant, split_k)
    return _linear("fp6_linear_fgq", need, X, hi, lo, scales, N, K, out, workspace, (variant, split_k), block=block)


# ---- FP5 E3M1 ("4+1")

def fp5_quantize_pack(W: torch.Tensor):
    """W fp16 [N,K] -> (hi_plane uint8 [N*K/2], lo_plane uint8 [N*K/8], scales fp16 [N])."""
    return _quantize_pack("fp5_quantize_pack", W, fp5_packed_sizes)


def fp5_unpack_codes(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int) -> torch.Tensor:
    return _unpack_codes("fp5_unpack_codes", hi, lo, N, K, 8)


def fp5_dequantize(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int) -> torch.Tensor:
    return _dequantize("fp5_dequantize", hi, lo, scales, N, K, 8)


def fp5_linear_workspace_bytes(M: int, N: int, K: int, variant: int = FP6_VARIANT_AUTO, split_k: int = 0) -> int:
    return int(lib().fp5_linear_workspace_bytes(M, N, K, variant, split_k))


def fp5_linear(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
               variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    need = lambda M: fp5_linear_workspace_bytes(M, N, K, variant, split_k)
    return _linear("fp5_linear", need, X, hi, lo, scales, N, K, out, workspace, (variant, split_k), lo_div=8)


# ---- FP6 in plane layout 2 (hardware conversion)

def fp6_quantize_pack_v2(W: torch.Tensor):
    return _quantize_pack("fp6_quantize_pack_v2", W, fp6_packed_sizes)


def fp6_unpack_codes_v2(hi: torch.Tensor, lo: torch.Tensor, N: int, K: int) -> torch.Tensor:
    return _unpack_codes("fp6_unpack_codes_v2", hi, lo, N, K, 4)


def fp6_dequantize_v2(hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int) -> torch.Tensor:
    return _dequantize("fp6_dequantize_v2", hi, lo, scales, N, K, 4)


def fp6_linear_v2_workspace_bytes(M: int, N: int, K: int, variant: int = FP6_VARIANT_AUTO, split_k: int = 0) -> int:
    return int(lib().fp6_linear_v2_workspace_bytes(M, N, K, variant, split_k))


def fp6_linear_v2(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                  variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    need = lambda M: fp6_linear_v2_workspace_bytes(M, N, K, variant, split_k)
    return _linear("fp6_linear_v2", need, X, hi, lo, scales, N, K, out, workspace, (variant, split_k))


def fp6_linear_v2_bf16(X: torch.Tensor, hi: torch.Tensor, lo: torch.Tensor, scales: torch.Tensor, N: int, K: int,
                       variant: int = FP6_VARIANT_AUTO, split_k: int = 0, out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Layout-2 planes against bf16 activations; returns bf16."""
    need = lambda M: fp6_linear_v2_workspace_bytes(M, N, K, variant, split_k)
    return _linear("fp6_linear_v2_bf16", need, X, hi, lo, scales, N, K, out, workspace, (variant, split_k),
                   dtype=torch.bfloat16)


# ---- measurement probes (kernels that only read, or only issue MFMAs)

def fp6_probe_read(buf: torch.Tensor, workgroups: int, sink: torch.Tensor) -> None:
    """One launch of the plain read kernel over all bytes of `buf` (a contiguous device tensor)."""
    if not (buf.is_cuda and buf.is_contiguous() and sink.is_cuda and sink.is_contiguous()):
        raise Fp6Error("buf and sink must be contiguous device tensors")
    _check(lib().fp6_probe_read(buf.data_ptr(), buf.numel() * buf.element_size(), workgroups, sink.data_ptr(),
                                sink.numel() * sink.element_size(), _stream()), "fp6_probe_read")


def fp6_probe_mfma(workgroups: int, iters: int, random_operands: bool, sink: torch.Tensor, wide: bool = False,
                   valu_mix: bool = False) -> int:
    """One launch of the MFMA-only kernel (valu_mix: with two integer vector instructions behind every MFMA);
    returns the flop count of the launch."""
    if not (sink.is_cuda and sink.is_contiguous()):
        raise Fp6Error("sink must be a contiguous device tensor")
    if wide and valu_mix:
        raise Fp6Error("the instruction mix exists for the 16x16x32 MFMA only")
    form = 2 if valu_mix else (1 if wide else 0)
    _check(lib().fp6_probe_mfma(workgroups, iters, int(bool(random_operands)), form, sink.data_ptr(),
                                sink.numel() * sink.element_size(), _stream()), "fp6_probe_mfma")
    return workgroups * 4 * 8 * iters * 16384 * (2 if wide else 1)
