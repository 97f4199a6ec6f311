"""GPU: nothing outside the buffers a call was given is written.

Every buffer of a call - Y, the workspace, both planes, the scales, X - is a window inside a larger
allocation whose surroundings (the guard bands) hold a poison pattern.  After the call the bands must
still hold the pattern byte for byte, and inputs must be unchanged.  Shapes are ragged in M and N and the
plans cover the streaming kernel (no split, pairwise meeting, counter meeting, half tiles, several row
blocks) and the tiled kernel (with and without split).  Y itself is still compared with the oracle."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from paper_2312_08583_amd import binding as B
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, oracle_reference

pytestmark = pytest.mark.gpu
DEV = "cuda"
BAND = 4096          # bytes of poison on each side (a multiple of 16: the windows stay aligned)
POISON = 0xA5


class Banded:
    """A contiguous window of `nbytes` bytes with poisoned guard bands before and after it."""

    def __init__(self, nbytes: int, fill=None):
        self.nbytes = nbytes
        self.raw = torch.full((nbytes + 2 * BAND,), POISON, dtype=torch.uint8, device=DEV)
        self.window = self.raw[BAND:BAND + nbytes]
        if fill is not None:
            self.window.copy_(fill.contiguous().view(torch.uint8).reshape(-1))

    def view(self, dtype, shape):
        return self.window.view(dtype).reshape(shape)

    def bands_intact(self) -> bool:
        return bool((self.raw[:BAND] == POISON).all()) and bool((self.raw[BAND + self.nbytes:] == POISON).all())


PLANS = [
    # (M, N, K, variant, split_k)
    (1, 192, 512, B.FP6_VARIANT_DECODE, 1),
    (3, 192, 512, B.FP6_VARIANT_DECODE, 2),                                   # two slices: pairwise slots
    (5, 320, 1536, B.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(1), 4),             # arrival counter + partial sums
    (2, 192, 1024, B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 1),             # half-tile workgroups, padded grid
    (4, 192, 1024, B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 2),
    (37, 192, 768, B.FP6_VARIANT_DECODE, 3),                                  # several row blocks per wavefront
    (37, 704, 512, B.FP6_VARIANT_GEMM, 1),                                    # ragged M, N not a multiple of 512
    (130, 704, 1024, B.FP6_VARIANT_GEMM | B.FP6_HINT_BLOCK_M(128), 2),
    (70, 320, 1024, B.FP6_VARIANT_GEMM | B.FP6_HINT_BLOCK_M(64) | B.FP6_HINT_WIDTH(4), 4),
    (1, 1024, 1024, B.FP6_VARIANT_AUTO, 0),
    (512, 1088, 512, B.FP6_VARIANT_AUTO, 0),
]


@pytest.mark.parametrize("M,N,K,variant,split", PLANS)
def test_linear_writes_only_inside_its_buffers(M, N, K, variant, split):
    W = inputs.weight(N, K, seed=700 + N + K, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=800 + M, device=DEV)
    hi0, lo0, sc0 = P.fp6_quantize_pack(W)
    hi, lo, sc = Banded(hi0.numel(), hi0), Banded(lo0.numel(), lo0), Banded(2 * N, sc0)
    xb = Banded(2 * M * K, X)
    yb = Banded(2 * M * N)
    yb.window.fill_(0x7E)                       # NaN patterns: every element of Y must be overwritten
    need = P.fp6_linear_variant_workspace_bytes(M, N, K, variant, split)
    ws = Banded(max(need, 16))
    ws.window.zero_()
    Y = yb.view(torch.float16, (M, N))
    for _ in range(2):                          # the second call finds the workspace as the first left it
        P.fp6_linear_variant(xb.view(torch.float16, (M, K)), hi.window, lo.window, sc.view(torch.float16, (N,)), N, K,
                             variant=variant, split_k=split, out=Y, workspace=ws.window if need else None)
    torch.cuda.synchronize()
    for name, b in (("Y", yb), ("workspace", ws), ("hi_plane", hi), ("lo_plane", lo), ("scales", sc), ("X", xb)):
        assert b.bands_intact(), "guard band of %s was written" % name
    assert torch.equal(hi.window, hi0) and torch.equal(lo.window, lo0), "planes were modified"
    assert torch.equal(sc.view(torch.float16, (N,)), sc0) and torch.equal(xb.view(torch.float16, (M, K)), X)
    if need:
        zero = min(need, B.FP6_WORKSPACE_ZERO_BYTES)
        assert not ws.window[:zero].any(), "counters and slots are not left zero"
    _, _, Yref = oracle_reference(W, X)
    assert_y_close(Y, Yref, "banded buffers")


@pytest.mark.parametrize("N,K,block", [(192, 320, 0), (64, 4096, 0), (320, 512, 128)])
def test_quantize_pack_and_utilities_write_only_inside_their_buffers(N, K, block):
    W = inputs.weight(N, K, seed=900 + N, sigma=0.02, outlier_frac=0.001, device=DEV)
    wb = Banded(2 * N * K, W)
    nscale = N * (K // block if block else 1)
    hi, lo, sc = Banded(N * K // 2), Banded(N * K // 4), Banded(2 * nscale)
    L, st = B.lib(), torch.cuda.current_stream().cuda_stream
    wp = wb.window.data_ptr()
    if block:
        rc = L.fp6_quantize_pack_fgq(wp, N, K, block, hi.window.data_ptr(), lo.window.data_ptr(), sc.window.data_ptr(), st)
    else:
        rc = L.fp6_quantize_pack(wp, N, K, hi.window.data_ptr(), lo.window.data_ptr(), sc.window.data_ptr(), st)
    assert rc == 0
    codes, what = Banded(N * K), Banded(2 * N * K)
    assert L.fp6_unpack_codes(hi.window.data_ptr(), lo.window.data_ptr(), N, K, codes.window.data_ptr(), st) == 0
    if block:
        rc = L.fp6_dequantize_fgq(hi.window.data_ptr(), lo.window.data_ptr(), sc.window.data_ptr(), N, K, block,
                                  what.window.data_ptr(), st)
    else:
        rc = L.fp6_dequantize(hi.window.data_ptr(), lo.window.data_ptr(), sc.window.data_ptr(), N, K, what.window.data_ptr(), st)
    assert rc == 0
    torch.cuda.synchronize()
    for name, b in (("W", wb), ("hi_plane", hi), ("lo_plane", lo), ("scales", sc), ("codes", codes), ("W_hat", what)):
        assert b.bands_intact(), "guard band of %s was written" % name
    assert torch.equal(wb.view(torch.float16, (N, K)), W)
    # and the windows hold what the ordinary call produces
    ref = P.fp6_quantize_pack_fgq(W, block) if block else P.fp6_quantize_pack(W)
    assert torch.equal(hi.window, ref[0]) and torch.equal(lo.window, ref[1])
    assert torch.equal(sc.view(torch.float16, ref[2].shape), ref[2])


def test_binding_rejects_buffers_that_do_not_match_the_shape():
    N, K, M = 128, 256, 4
    W = inputs.weight(N, K, seed=5, device=DEV)
    X = inputs.activation(M, K, seed=6, device=DEV)
    hi, lo, sc = P.fp6_quantize_pack(W)
    with pytest.raises(P.Fp6Error):
        P.fp6_linear(X, hi[:-16], lo, sc, N, K)
    with pytest.raises(P.Fp6Error):
        P.fp6_linear(X, hi, lo[:-16], sc, N, K)
    with pytest.raises(P.Fp6Error):
        P.fp6_linear(X, hi, lo, sc[:-1], N, K)
    with pytest.raises(P.Fp6Error):
        P.fp6_linear(X, hi, lo, sc, N, K, out=torch.empty((M, N + 64), dtype=torch.float16, device=DEV))
    with pytest.raises(P.Fp6Error):
        P.fp6_linear(X, hi, lo, sc, 2 * N, K)                 # planes too small for the N that is claimed
    with pytest.raises(P.Fp6Error):
        P.fp6_linear(X[:, :K - 64].contiguous(), hi, lo, sc, N, K)
    with pytest.raises(P.Fp6Error):
        P.fp5_linear(X, hi, lo, sc, N, K)                     # a 2-bit plane is not a 1-bit plane
    with pytest.raises(P.Fp6Error):
        P.fp6_linear_fgq(X, hi, lo, sc, N, K, 64)             # row scales are not block scales
    with pytest.raises(P.Fp6Error):
        P.fp6_dequantize(hi, lo, sc, N, 2 * K)
    Y = P.fp6_linear(X, hi, lo, sc, N, K)                     # the matching call still works
    torch.cuda.synchronize()
    assert torch.isfinite(Y).all()
