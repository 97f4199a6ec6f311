"""GPU parity of the fine-grained (block-k scale) calls against the CPU oracle: scales,
codes, planes and dequantized weights bit-exact; Y within 2e-3 (gpu_util.assert_y_close).
The library keeps scales block-major ([K/block, N]); the oracle's logical shape is [N, K/block]."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from oracle import fp6_oracle as O
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, from_np16, to_np16
from layout_ref import pack_planes

pytestmark = pytest.mark.gpu
DEV = "cuda"
B = P.binding


def _quant(W, block):
    hi, lo, sc = P.fp6_quantize_pack_fgq(W, block)
    torch.cuda.synchronize()
    return hi, lo, sc


@pytest.mark.parametrize("block", [64, 128, 256, 512])
def test_fgq_quantize_pack_bit_exact(block):
    N, K = 192, 1024
    W = inputs.weight(N, K, seed=1200 + block, sigma=0.02, outlier_frac=0.001, device=DEV)
    W[5, 128:256] = 0                                    # a block of zeros: S = 0, signed-zero codes
    W[7, 0:64] = -W[7, 0:64].abs() * 1e-4                # tiny negatives
    hi, lo, sc = _quant(W, block)
    codes_o, scales_o = O.quantize_fgq(to_np16(W), block)
    assert np.array_equal(to_np16(sc), scales_o.T)
    assert np.array_equal(P.fp6_unpack_codes(hi, lo, N, K).cpu().numpy(), codes_o)
    hi_o, lo_o = pack_planes(codes_o)
    assert np.array_equal(hi.cpu().numpy(), hi_o) and np.array_equal(lo.cpu().numpy(), lo_o)
    what = to_np16(P.fp6_dequantize_fgq(hi, lo, sc, N, K, block))
    assert np.array_equal(what, O.dequantize_fgq(codes_o, scales_o, block))


def test_fgq_with_block_k_equals_the_row_wise_calls():
    N, K = 128, 512
    W = inputs.weight(N, K, seed=1300, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(5, K, seed=1301, device=DEV)
    hi, lo, sc = _quant(W, K)
    hi2, lo2, sc2 = P.fp6_quantize_pack(W)
    assert torch.equal(hi, hi2) and torch.equal(lo, lo2) and torch.equal(sc.reshape(-1), sc2)
    Ya = P.fp6_linear_fgq(X, hi, lo, sc, N, K, K)
    Yb = P.fp6_linear(X, hi2, lo2, sc2, N, K)
    torch.cuda.synchronize()
    # same numbers; the fine-grained path applies the scale tile by tile, so only the fp32 rounding differs
    Yref = O.linear(to_np16(X), *O.quantize(to_np16(W)))
    assert_y_close(Ya, Yref, "fgq block=K")
    assert (Ya.float() - Yb.float()).abs().max().item() <= 1e-3 * Yb.float().abs().max().item()


@pytest.mark.parametrize("block", [64, 128, 256])
@pytest.mark.parametrize("M,variant,split", [(1, B.FP6_VARIANT_DECODE, 1), (3, B.FP6_VARIANT_DECODE, 2),
                                             (16, B.FP6_VARIANT_DECODE, 4), (1, B.FP6_VARIANT_DECODE, 0),
                                             (17, B.FP6_VARIANT_GEMM, 1), (40, B.FP6_VARIANT_GEMM, 2),
                                             (100, B.FP6_VARIANT_GEMM, 1), (100, B.FP6_VARIANT_GEMM, 3),
                                             (8, B.FP6_VARIANT_GEMM, 1), (300, B.FP6_VARIANT_AUTO, 0),
                                             (40, B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(4) | B.FP6_HINT_BLOCK_M(32), 2),
                                             (100, B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(4) | B.FP6_HINT_BLOCK_M(64), 3),
                                             (100, B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(8) | B.FP6_HINT_BLOCK_M(64), 1)])
def test_fgq_linear_vs_oracle(block, M, variant, split):
    N, K = 640, 1536
    W = inputs.weight(N, K, seed=1400 + block, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=1410 + M, device=DEV)
    hi, lo, sc = _quant(W, block)
    codes_o, scales_o = O.quantize_fgq(to_np16(W), block)
    Yref = O.linear_fgq(to_np16(X), codes_o, scales_o, block)
    Y = P.fp6_linear_fgq(X, hi, lo, sc, N, K, block, variant, split)
    torch.cuda.synchronize()
    assert_y_close(Y, Yref, (block, M, variant, split))


@pytest.mark.parametrize("variant", [B.FP6_VARIANT_DECODE, B.FP6_VARIANT_GEMM])
def test_fgq_one_hot_rows_read_back_dequantized_weights_bit_exact(variant):
    # X one-hot: Y[m, n] = RNE_fp16(S[n, k_m / block] * value(code[n, k_m])) exactly; the scales
    # differ from block to block, so a scale taken from the wrong block shows
    N, K, block = 128, 512, 64
    rng = np.random.default_rng(77)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    hi, lo = pack_planes(codes)
    scales = (0.004 + 0.046 * rng.random((N, K // block))).astype(np.float16).view(np.uint16)
    what = O.dequantize_fgq(codes, scales, block)
    what = np.where((what & 0x7FFF) == 0, 0, what).astype(np.uint16)      # a sum that starts at +0 cannot give -0
    hi_d, lo_d = torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV)
    sc_d = from_np16(np.ascontiguousarray(scales.T))
    cols = [0, 63, 64, 127, 130, 200, 255, 256, 300, 383, 384, 447, 448, 500, 510, 511]
    X = torch.zeros((len(cols), K), dtype=torch.float16, device=DEV)
    for m, k in enumerate(cols):
        X[m, k] = 1.0
    if variant == B.FP6_VARIANT_GEMM:
        X = torch.cat([X, X, X[:1]])
    Y = to_np16(P.fp6_linear_fgq(X, hi_d, lo_d, sc_d, N, K, block, variant, 1))
    Y = np.where((Y & 0x7FFF) == 0, 0, Y).astype(np.uint16)
    for m, k in enumerate(cols):
        assert np.array_equal(Y[m], what[:, k]), (m, k)


def test_fgq_argument_errors():
    N, K = 128, 384
    W = inputs.weight(N, K, seed=1, device=DEV)
    with pytest.raises(P.Fp6Error):
        P.fp6_quantize_pack_fgq(W, 192)                    # 3 * 64: not 64 times a power of two
    with pytest.raises(P.Fp6Error):
        P.fp6_quantize_pack_fgq(W, 256)                    # does not divide K
    hi, lo, sc = _quant(W, 128)
    X = inputs.activation(2, K, seed=2, device=DEV)
    with pytest.raises(P.Fp6Error):
        P.fp6_linear_fgq(X, hi, lo, sc, N, K, 128, B.FP6_VARIANT_DECODE | B.FP6_HINT_DEQUANT(1), 1)
