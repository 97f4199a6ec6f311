"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol
the header declares, and rejects bad arguments before anything is launched.  Also the
host-side argument that the kernels' fp32 arithmetic decides exactly like real
arithmetic (checked against the oracle with numpy float32 standing in for the GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import fp6_oracle as O
from paper_2312_08583_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fp6_linear.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(fp[56]_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.fp6_layout_version() == 1


def test_packed_sizes_are_three_quarters_of_a_byte_per_weight():
    for N, K in [(64, 64), (1024, 1024), (4096, 11008), (28672, 8192), (5504, 2048)]:
        hi, lo, sc = B.fp6_packed_sizes(N, K)
        assert (hi, lo, sc) == (N * K // 2, N * K // 4, 2 * N)
        assert 4 * (hi + lo) == 3 * N * K          # 0.75 B per weight (4+2 bits)
    L = B.lib()
    for N, K in [(0, 64), (64, 0), (-64, 64), (63, 64), (64, 100), (1 << 31, 64)]:
        assert L.fp6_packed_sizes(N, K, None, None, None) == -2


def test_status_strings():
    seen = set()
    for st in range(0, -8, -1):
        s = B.fp6_status_string(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert B.fp6_status_string(-99) == "unknown status"


def test_argument_errors_are_reported_without_a_gpu():
    L = B.lib()
    buf = ctypes.create_string_buffer(1 << 16)
    a = (ctypes.addressof(buf) + 15) & ~15          # an aligned, non-device address: never dereferenced
    null = None
    # NULL pointers
    assert L.fp6_quantize_pack(null, 64, 64, a, a, a, None) == -1
    assert L.fp6_unpack_codes(a, null, 64, 64, a, None) == -1
    assert L.fp6_dequantize(a, a, null, 64, 64, a, None) == -1
    assert L.fp6_linear(a, 1, a, a, a, 64, 64, null, None, 0, None) == -1
    # shapes
    assert L.fp6_quantize_pack(a, 65, 64, a, a, a, None) == -2
    assert L.fp6_linear(a, 0, a, a, a, 64, 64, a, None, 0, None) == -2
    assert L.fp6_linear(a, 1, a, a, a, 64, 96, a, None, 0, None) == -2
    assert L.fp6_linear(a, -3, a, a, a, 64, 64, a, None, 0, None) == -2
    # alignment
    assert L.fp6_linear(a + 2, 1, a, a, a, 64, 64, a, None, 0, None) == -3
    assert L.fp6_dequantize(a, a + 8, a, 64, 64, a, None) == -3
    # variant / split requests
    assert L.fp6_linear_variant(a, 65, a, a, a, 64, 64, a, None, 0, None, B.FP6_VARIANT_DECODE, 0) == -5
    assert L.fp6_linear_variant(a, 1, a, a, a, 64, 256, a, None, 0, None, B.FP6_VARIANT_DECODE, 3) == -5
    assert L.fp6_linear_variant(a, 1, a, a, a, 64, 256, a, None, 0, None, 7, 0) == -5
    # workspace: a split needs one
    need = B.fp6_linear_variant_workspace_bytes(1, 64, 256, B.FP6_VARIANT_DECODE, 2)
    assert need >= B.FP6_WORKSPACE_ZERO_BYTES
    assert L.fp6_linear_variant(a, 1, a, a, a, 64, 256, a, None, 0, None, B.FP6_VARIANT_DECODE, 2) == -4
    assert L.fp6_linear_variant(a, 1, a, a, a, 64, 256, a, a, need - 1, None, B.FP6_VARIANT_DECODE, 2) == -4


def test_workspace_bytes():
    assert B.fp6_linear_variant_workspace_bytes(1, 64, 64, B.FP6_VARIANT_DECODE, 1) == 0
    # small M: the slices meet pairwise inside the zero region; at a counter they need a buffer
    assert B.fp6_linear_variant_workspace_bytes(1, 1024, 1024, B.FP6_VARIANT_DECODE, 2) == B.FP6_WORKSPACE_ZERO_BYTES
    assert B.fp6_linear_variant_workspace_bytes(1, 1024, 1024, B.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(2), 4) == \
        B.FP6_WORKSPACE_ZERO_BYTES
    assert B.fp6_linear_variant_workspace_bytes(1, 1024, 1024, B.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(1), 4) == \
        B.FP6_WORKSPACE_ZERO_BYTES + 4 * 16 * 64 * 16 * 4
    assert B.fp6_linear_variant_workspace_bytes(16, 1024, 1024, B.FP6_VARIANT_DECODE, 4) == \
        B.FP6_WORKSPACE_ZERO_BYTES + 4 * 16 * 64 * 16 * 4
    # pairwise meeting that does not fit the slot region is refused
    assert B.fp6_linear_variant_workspace_bytes(16, 32768, 8192, B.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(2), 4) == 0
    assert B.fp6_linear_variant_workspace_bytes(100, 512, 1024, B.FP6_VARIANT_GEMM, 2) == \
        B.FP6_WORKSPACE_ZERO_BYTES + 2 * 2 * 128 * 256 * 4
    assert B.fp6_linear_workspace_bytes(0, 64, 64) == 0          # invalid shapes need nothing
    for M, N, K in [(1, 4096, 4096), (16, 8192, 28672), (512, 8192, 28672), (128, 5120, 13824)]:
        assert B.fp6_linear_workspace_bytes(M, N, K) % 16 == 0


def test_plan_query_agrees_with_the_calls_it_describes():
    """fp6_linear_plan runs the planner of the hot-path calls: its workspace size is theirs, its launch is
    consistent, and the families sit where the design puts them (decode up to 16 rows, tiled from 128 on)."""
    from paper_2312_08583_amd import inputs
    seen = set()
    for wl, cfg in inputs.WORKLOADS.items():
        for (_, N, K) in cfg["shapes"]:
            for M in sorted(set(cfg["Ms"]) | {1, 3, 16, 17, 40, 64, 100, 512}):
                p = B.fp6_linear_plan(M, N, K)
                assert p["workspace_bytes"] == B.fp6_linear_workspace_bytes(M, N, K)
                assert p["variant"] in (B.FP6_VARIANT_DECODE, B.FP6_VARIANT_GEMM)
                assert p["split_k"] >= 1 and (K // 64) % p["split_k"] == 0
                assert (p["meeting"] == 0) == (p["split_k"] == 1)
                assert (p["workspace_bytes"] == 0) == (p["split_k"] == 1)
                assert p["workgroups"] >= 1
                if M <= 16:
                    assert p["variant"] == B.FP6_VARIANT_DECODE and p["block_m"] == 16
                if M >= 128:
                    assert p["variant"] == B.FP6_VARIANT_GEMM and p["block_m"] in (32, 64, 128) and p["width"] in (4, 8)
                if p["variant"] == B.FP6_VARIANT_DECODE:
                    per = (N // 64) * p["split_k"]
                    assert p["workgroups"] == ((per + 7) // 8 * 16 if p["half_tiles"] else per)
                    assert M <= p["block_m"]
                else:
                    mblk = -(-M // p["block_m"])
                    nblk = -(-(N // 64) // p["width"])
                    assert p["workgroups"] == mblk * ((nblk * p["split_k"] + 7) // 8 * 8)
                seen.add(p["variant"])
                # a forced plan is reported as forced
                q = B.fp6_linear_plan(M, N, K, variant=B.FP6_VARIANT_GEMM | B.FP6_HINT_BLOCK_M(32), split_k=1)
                assert (q["variant"], q["block_m"], q["split_k"], q["meeting"]) == (B.FP6_VARIANT_GEMM, 32, 1, 0)
                # the other formats and fine-grained scales plan too
                for fmt in (B.FP6_FORMAT_E3M1, B.FP6_FORMAT_E3M2_V2, B.FP6_FORMAT_E3M2_V2_BF16):
                    assert B.fp6_linear_plan(M, N, K, format=fmt)["workgroups"] >= 1
                assert B.fp6_linear_plan(M, N, K, block=64)["workspace_bytes"] == B.fp6_linear_fgq_workspace_bytes(M, N, K, 64)
    assert seen == {B.FP6_VARIANT_DECODE, B.FP6_VARIANT_GEMM}
    L = B.lib()
    info = B.PlanInfo()
    assert L.fp6_linear_plan(6, 1, 64, 64, 0, 0, 0, None) == -1
    assert L.fp6_linear_plan(6, 0, 64, 64, 0, 0, 0, ctypes.byref(info)) == -2
    assert L.fp6_linear_plan(6, 1, 64, 100, 0, 0, 0, ctypes.byref(info)) == -2
    assert L.fp6_linear_plan(9, 1, 64, 64, 0, 0, 0, ctypes.byref(info)) == -5
    assert L.fp6_linear_plan(6, 65, 64, 64, 0, B.FP6_VARIANT_DECODE, 0, ctypes.byref(info)) == -5
    assert L.fp6_linear_plan(6, 1, 64, 256, 96, 0, 0, ctypes.byref(info)) == -5          # block not 64 * 2^j


def test_no_cpu_fallback():
    import torch
    W = torch.zeros((64, 64), dtype=torch.float16)
    with pytest.raises(B.Fp6Error):
        B.fp6_quantize_pack(W)


# ---------------------------------------------------------------------------
# The GPU quantizer divides in fp32 (one IEEE division, then one rounding) instead of in
# exact arithmetic.  numpy float32 has the same IEEE semantics, so the claim that this
# decides identically can be checked on the host against the oracle, exhaustively.

def _scale_fp32(amax16: np.ndarray) -> np.ndarray:
    return (amax16.astype(np.float32) / np.float32(28.0)).astype(np.float16)


def _codes_fp32(w16: np.ndarray, S16: np.float16) -> np.ndarray:
    """The quantizer kernel's arithmetic, operation by operation, in numpy float32 / uint32."""
    sign = (w16.view(np.uint16) >> 15).astype(np.uint8) << 5
    S = np.float32(S16)
    if S == 0:
        return sign
    q = np.minimum(np.abs(w16).astype(np.float32) / S, np.float32(28.0))
    b = q.view(np.uint32)
    top = (b + np.uint32((1 << 20) - 1) + ((b >> 21) & 1)) >> 21          # nearest even on the bit pattern
    normal = top - np.uint32(124 << 2)
    t = (q + np.float32(1 << 19)).astype(np.float32)                       # multiples of 1/16, nearest even
    sub = t.view(np.uint32) & 7
    return sign | np.where(q < np.float32(0.25), sub, normal).astype(np.uint8)


def test_fp32_scale_division_matches_exact_for_every_amax():
    amax = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16)
    got = _scale_fp32(amax).view(np.uint16)
    want = np.array([O.row_scale(np.array([b], np.uint16)) for b in range(0, 0x7C00)], np.uint16)
    assert np.array_equal(got, want)


def test_fp32_code_rounding_matches_exact_for_every_weight_and_many_scales():
    allw = np.arange(0, 0x7C00, dtype=np.uint16)
    rng = np.random.default_rng(2)
    amax_bits = [0x3C00, 0x2E66, 0x2C00, 0x3555, 0x0155, 0x0400, 0x7BFF, 0x1234] + \
        rng.integers(0x0400, 0x7BFF, 12).tolist()
    for ab in amax_bits:
        w = allw[allw <= ab]
        row = np.concatenate([w, w | 0x8000]).astype(np.uint16)
        codes, scales = O.quantize(row[None, :])
        S16 = scales.view(np.float16)[0]
        assert _scale_fp32(np.array([ab], np.uint16).view(np.float16))[0] == S16
        got = _codes_fp32(row.view(np.float16), S16)
        assert np.array_equal(got, codes[0]), hex(ab)
