"""GPU parity of the FP5 E3M1 ("4+1") calls against the CPU oracle: scales, codes, planes and
dequantized weights bit-exact; Y within 2e-3 (gpu_util.assert_y_close)."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from oracle import fp6_oracle as O
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, from_np16, to_np16
from layout_ref import pack_planes5

pytestmark = pytest.mark.gpu
DEV = "cuda"
B = P.binding


def _check_quant(Wnp16):
    N, K = Wnp16.shape
    hi, lo, sc = P.fp5_quantize_pack(from_np16(Wnp16))
    torch.cuda.synchronize()
    codes_o, scales_o = O.quantize5(Wnp16)
    assert np.array_equal(to_np16(sc), scales_o)
    assert np.array_equal(P.fp5_unpack_codes(hi, lo, N, K).cpu().numpy(), codes_o)
    hi_o, lo_o = pack_planes5(codes_o)
    assert hi.numel() == N * K // 2 and lo.numel() == N * K // 8          # 0.625 byte per weight
    assert np.array_equal(hi.cpu().numpy(), hi_o) and np.array_equal(lo.cpu().numpy(), lo_o)
    assert np.array_equal(to_np16(P.fp5_dequantize(hi, lo, sc, N, K)), O.dequantize5(codes_o, scales_o))
    return hi, lo, sc, codes_o, scales_o


def test_fp5_quantize_pack_bit_exact_on_workload_like_weights():
    W = inputs.weight(256, 1024, seed=1500, sigma=0.02, outlier_frac=0.001, device=DEV)
    W[3] = 0
    W[9, :64] = -W[9, :64].abs() * 1e-4
    _check_quant(to_np16(W))


def test_fp5_quantize_every_finite_fp16_value_at_many_scales():
    # rows that together hold every finite fp16 magnitude up to amax, for several amax (scales with
    # odd significands, a power of two, a subnormal scale): every rounding decision, ties included
    for amax_bits in (0x3C00, 0x2E66, 0x3555, 0x1234, 0x0280, 0x57FF):
        vals = np.arange(0, amax_bits + 1, dtype=np.uint16)
        K = 64 * ((vals.size + 63) // 64 + 1)
        row = np.full(K, amax_bits, np.uint16)
        row[:vals.size] = vals
        row[1::2] |= 0x8000                                  # alternate signs
        _check_quant(np.tile(row, (64, 1)))


def test_fp5_planes_round_trip_for_arbitrary_codes():
    rng = np.random.default_rng(3)
    N, K = 128, 256
    codes = rng.integers(0, 32, (N, K), dtype=np.uint8)
    hi, lo = pack_planes5(codes)
    got = P.fp5_unpack_codes(torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), N, K).cpu().numpy()
    assert np.array_equal(got, codes)
    hi4, lo1 = O.split41(codes)
    assert np.array_equal(hi4, got >> 1) and np.array_equal(lo1, got & 1)


@pytest.mark.parametrize("variant,split", [(B.FP6_VARIANT_DECODE, 1), (B.FP6_VARIANT_DECODE, 2),
                                           (B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 1),
                                           (B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 2),
                                           (B.FP6_VARIANT_GEMM, 1), (B.FP6_VARIANT_GEMM, 2),
                                           (B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(4), 2)])
def test_fp5_one_hot_rows_read_back_dequantized_weights_bit_exact(variant, split):
    N, K = 128, 256
    rng = np.random.default_rng(13)
    codes = rng.integers(0, 32, (N, K), dtype=np.uint8)
    codes[:, :32] = np.arange(32, dtype=np.uint8)[None, :]
    hi, lo = pack_planes5(codes)
    scales = np.linspace(0.004, 0.05, N).astype(np.float16).view(np.uint16)
    what = O.dequantize5(codes, scales)
    what = np.where((what & 0x7FFF) == 0, 0, what).astype(np.uint16)
    hi_d, lo_d, sc_d = torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), from_np16(scales)
    ks = list(range(32)) + [100, 255, 128, 191] + list(range(64, 76))
    for k0 in range(0, len(ks), 16):
        cols = ks[k0:k0 + 16]
        X = torch.zeros((len(cols), K), dtype=torch.float16, device=DEV)
        for m, k in enumerate(cols):
            X[m, k] = 1.0
        if (variant & 0xFF) == B.FP6_VARIANT_GEMM:
            X = torch.cat([X, X, X[:1]])
        Y = to_np16(P.fp5_linear(X, hi_d, lo_d, sc_d, N, K, variant, split))
        Y = np.where((Y & 0x7FFF) == 0, 0, Y).astype(np.uint16)
        for m, k in enumerate(cols):
            assert np.array_equal(Y[m], what[:, k]), (m, k)


@pytest.mark.parametrize("M,variant,split", [(1, B.FP6_VARIANT_AUTO, 0), (1, B.FP6_VARIANT_DECODE, 1),
                                             (7, B.FP6_VARIANT_DECODE, 4), (16, B.FP6_VARIANT_DECODE, 3),
                                             (17, B.FP6_VARIANT_GEMM, 1), (40, B.FP6_VARIANT_GEMM, 2),
                                             (100, B.FP6_VARIANT_GEMM, 1), (300, B.FP6_VARIANT_AUTO, 0),
                                             (1, B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 1),
                                             (3, B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 2),
                                             (4, B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1), 4),
                                             (16, B.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1) | B.FP6_HINT_MEET(1), 2),
                                             (70, B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(4) | B.FP6_HINT_BLOCK_M(64), 3),
                                             (130, B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(4) | B.FP6_HINT_BLOCK_M(128), 2)])
def test_fp5_linear_vs_oracle(M, variant, split):
    N, K = 640, 1536
    W = inputs.weight(N, K, seed=1600, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=1610 + M, device=DEV)
    hi, lo, sc = P.fp5_quantize_pack(W)
    codes_o, scales_o = O.quantize5(to_np16(W))
    Yref = O.linear5(to_np16(X), codes_o, scales_o)
    Y = P.fp5_linear(X, hi, lo, sc, N, K, variant, split)
    torch.cuda.synchronize()
    assert_y_close(Y, Yref, (M, variant, split))


def test_fp5_rejects_hints_it_does_not_have():
    N, K = 128, 256
    W = inputs.weight(N, K, seed=1, device=DEV)
    hi, lo, sc = P.fp5_quantize_pack(W)
    X = inputs.activation(1, K, seed=2, device=DEV)
    with pytest.raises(P.Fp6Error):
        P.fp5_linear(X, hi, lo, sc, N, K, B.FP6_VARIANT_DECODE | B.FP6_HINT_DEQUANT(1), 1)
