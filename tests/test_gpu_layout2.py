"""GPU parity of the FP6 calls in plane layout 2 (planes that merge into the operand of gfx950's packed
E3M2 -> fp16 conversion): scales, codes, planes and dequantized weights bit-exact against the oracle and
the numpy statement of the layout; Y within 2e-3 (gpu_util.assert_y_close)."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from oracle import fp6_oracle as O
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, from_np16, to_np16
from layout_ref import pack_planes_v2

pytestmark = pytest.mark.gpu
DEV = "cuda"
B = P.binding


def test_layout2_quantize_pack_bit_exact():
    N, K = 128, 256
    W = inputs.weight(N, K, seed=2500, sigma=0.02, outlier_frac=0.002, device=DEV)
    W[3] = 0
    W[9, :64] = -W[9, :64].abs() * 1e-4
    hi, lo, sc = P.fp6_quantize_pack_v2(W)
    torch.cuda.synchronize()
    codes_o, scales_o = O.quantize(to_np16(W))
    assert np.array_equal(to_np16(sc), scales_o)
    assert np.array_equal(P.fp6_unpack_codes_v2(hi, lo, N, K).cpu().numpy(), codes_o)
    hi_o, lo_o = pack_planes_v2(codes_o)
    assert np.array_equal(hi.cpu().numpy(), hi_o) and np.array_equal(lo.cpu().numpy(), lo_o)
    assert np.array_equal(to_np16(P.fp6_dequantize_v2(hi, lo, sc, N, K)), O.dequantize(codes_o, scales_o))
    # same scales and codes as layout 1; the planes differ
    hi1, lo1, sc1 = P.fp6_quantize_pack(W)
    assert torch.equal(sc, sc1) and not torch.equal(hi, hi1)


def test_layout2_planes_round_trip_and_keep_the_4_plus_2_split():
    rng = np.random.default_rng(4)
    N, K = 64, 128
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    hi, lo = pack_planes_v2(codes)
    got = P.fp6_unpack_codes_v2(torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), N, K).cpu().numpy()
    assert np.array_equal(got, codes)
    # the 2-bit plane depends on the mantissas only, the 4-bit plane on sign and exponent only (Section 5.1)
    hi_m, lo_m = pack_planes_v2(codes & 3)
    hi_s, lo_s = pack_planes_v2(codes & 0x3C)
    assert not hi_m.any() and np.array_equal(lo_m, lo)
    assert not lo_s.any() and np.array_equal(hi_s, hi)


@pytest.mark.parametrize("variant,split", [(B.FP6_VARIANT_DECODE, 1), (B.FP6_VARIANT_DECODE, 2),
                                           (B.FP6_VARIANT_GEMM, 1), (B.FP6_VARIANT_GEMM, 2)])
def test_layout2_one_hot_rows_read_back_dequantized_weights_bit_exact(variant, split):
    # through the hardware conversion: every code, FP6 subnormals and -0 included
    N, K = 128, 256
    rng = np.random.default_rng(14)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    codes[:, :64] = np.arange(64, dtype=np.uint8)[None, :]
    hi, lo = pack_planes_v2(codes)
    scales = np.linspace(0.004, 0.05, N).astype(np.float16).view(np.uint16)
    what = O.dequantize(codes, scales)
    what = np.where((what & 0x7FFF) == 0, 0, what).astype(np.uint16)
    hi_d, lo_d, sc_d = torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), from_np16(scales)
    ks = list(range(64)) + [100, 255, 128, 191] + list(range(64, 76))
    for k0 in range(0, len(ks), 16):
        cols = ks[k0:k0 + 16]
        X = torch.zeros((len(cols), K), dtype=torch.float16, device=DEV)
        for m, k in enumerate(cols):
            X[m, k] = 1.0
        if variant == B.FP6_VARIANT_GEMM:
            X = torch.cat([X, X, X[:1]])
        Y = to_np16(P.fp6_linear_v2(X, hi_d, lo_d, sc_d, N, K, variant, split))
        Y = np.where((Y & 0x7FFF) == 0, 0, Y).astype(np.uint16)
        for m, k in enumerate(cols):
            assert np.array_equal(Y[m], what[:, k]), (m, k)


@pytest.mark.parametrize("M,variant,split", [(1, B.FP6_VARIANT_AUTO, 0), (7, B.FP6_VARIANT_DECODE, 4),
                                             (16, B.FP6_VARIANT_DECODE, 3), (17, B.FP6_VARIANT_GEMM, 1),
                                             (40, B.FP6_VARIANT_GEMM, 2), (100, B.FP6_VARIANT_GEMM, 1),
                                             (300, B.FP6_VARIANT_AUTO, 0)])
def test_layout2_linear_vs_oracle(M, variant, split):
    N, K = 640, 1536
    W = inputs.weight(N, K, seed=2600, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=2610 + M, device=DEV)
    hi, lo, sc = P.fp6_quantize_pack_v2(W)
    codes_o, scales_o = O.quantize(to_np16(W))
    Yref = O.linear(to_np16(X), codes_o, scales_o)
    Y = P.fp6_linear_v2(X, hi, lo, sc, N, K, variant, split)
    torch.cuda.synchronize()
    assert_y_close(Y, Yref, (M, variant, split))


# ---- bf16 activations on the planes of layout 2 (fp6_linear_v2_bf16)

def _bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _assert_close_bf16(Y: torch.Tensor, Yref: np.ndarray, what=""):
    """bf16 keeps 8 significant bits: rounding the result to it costs up to 2^-8 = 3.9e-3 of |y| (half a unit
    in the last place), eight times the fp16 figure, so the 2e-3 bar of the fp16 path cannot apply.  The bar
    here: element-wise |Y - Yref| <= 2^-8 |Yref| (the output rounding) + 1e-4 (|Yref| + rms(Yref)) (fp32
    accumulation, measured ~1e-5), which also bounds max|Y - Yref| / max|Yref| by 4.1e-3."""
    assert torch.isfinite(Y).all(), what
    y = Y.detach().cpu().to(torch.float64).numpy()
    err = np.abs(y - Yref)
    rms = np.sqrt(np.mean(Yref ** 2))
    excess = (err - (2.0 ** -8 * np.abs(Yref) + 1e-4 * (np.abs(Yref) + rms))).max()
    assert excess <= 0, (what, excess)
    assert err.max() / np.abs(Yref).max() <= 4.1e-3, what


@pytest.mark.parametrize("variant,split", [(B.FP6_VARIANT_DECODE, 1), (B.FP6_VARIANT_DECODE, 2),
                                           (B.FP6_VARIANT_GEMM, 1), (B.FP6_VARIANT_GEMM, 2)])
def test_bf16_one_hot_rows_read_back_the_weights_rounded_to_bf16_bit_exact(variant, split):
    # Y[m][n] = bf16_RNE(S_n * v(c[n][k_m])): every code through the bf16 form of the hardware conversion,
    # FP6 subnormals and -0 included; the product S * v is exact in fp32, so one rounding decides
    N, K = 128, 256
    rng = np.random.default_rng(15)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    codes[:, :64] = np.arange(64, dtype=np.uint8)[None, :]
    hi, lo = pack_planes_v2(codes)
    scales = np.linspace(0.004, 0.05, N).astype(np.float16)
    Sv = scales.astype(np.float64)[:, None] * np.array([[O.e3m2_value(int(c)) for c in row] for row in codes])
    want = np.array([[O.double_to_bf16(float(v)) for v in row] for row in Sv], dtype=np.uint16)
    want = np.where((want & 0x7FFF) == 0, 0, want).astype(np.uint16)
    hi_d, lo_d, sc_d = torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), from_np16(scales.view(np.uint16))
    ks = list(range(64)) + [100, 255, 128, 191] + list(range(64, 76))
    for k0 in range(0, len(ks), 16):
        cols = ks[k0:k0 + 16]
        X = torch.zeros((len(cols), K), dtype=torch.bfloat16, device=DEV)
        for m, k in enumerate(cols):
            X[m, k] = 1.0
        if variant == B.FP6_VARIANT_GEMM:
            X = torch.cat([X, X, X[:1]])
        Y = _bf16_bits(P.fp6_linear_v2_bf16(X, hi_d, lo_d, sc_d, N, K, variant, split))
        Y = np.where((Y & 0x7FFF) == 0, 0, Y).astype(np.uint16)
        for m, k in enumerate(cols):
            assert np.array_equal(Y[m], want[:, k]), (m, k)


@pytest.mark.parametrize("M,variant,split", [(1, B.FP6_VARIANT_AUTO, 0), (7, B.FP6_VARIANT_DECODE, 4),
                                             (16, B.FP6_VARIANT_DECODE, 3), (17, B.FP6_VARIANT_GEMM, 1),
                                             (40, B.FP6_VARIANT_GEMM, 2), (100, B.FP6_VARIANT_GEMM, 1),
                                             (130, B.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(4) | B.FP6_HINT_BLOCK_M(128), 2),
                                             (300, B.FP6_VARIANT_AUTO, 0)])
def test_bf16_linear_vs_oracle(M, variant, split):
    N, K = 640, 1536
    W = inputs.weight(N, K, seed=2700, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation_bf16(M, K, seed=2710 + M, device=DEV)
    hi, lo, sc = P.fp6_quantize_pack_v2(W)
    codes_o, scales_o = O.quantize(to_np16(W))
    Yref = O.linear_bf16(_bf16_bits(X), codes_o, scales_o)
    ws = P.new_workspace(max(16, P.fp6_linear_v2_workspace_bytes(M, N, K, variant, split)), DEV)
    Y = P.fp6_linear_v2_bf16(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    torch.cuda.synchronize()
    assert Y.dtype == torch.bfloat16
    _assert_close_bf16(Y, Yref, (M, variant, split))
    assert torch.count_nonzero(ws[:B.FP6_WORKSPACE_ZERO_BYTES]).item() == 0 or ws.numel() < B.FP6_WORKSPACE_ZERO_BYTES


@pytest.mark.parametrize("M", [1, 512])
def test_bf16_full_size_shape_sampled(M):
    # gate projection of the benchmark stack, automatic plan, sampled channels
    N, K = 22016, 8192
    W = inputs.workload_weight("cfg5_34b_stack", 4, layer=1, device=DEV)
    X = inputs.activation_bf16(M, K, seed=2800 + M, device=DEV)
    hi, lo, sc = P.fp6_quantize_pack_v2(W)
    rows = np.sort(np.random.default_rng(5).choice(N, size=192, replace=False))
    rows[0], rows[-1] = 0, N - 1
    ridx = torch.from_numpy(rows).to(DEV)
    codes_o, scales_o = O.quantize(to_np16(W[ridx]))
    Y = P.fp6_linear_v2_bf16(X, hi, lo, sc, N, K)
    torch.cuda.synchronize()
    _assert_close_bf16(Y[:, ridx], O.linear_bf16(_bf16_bits(X), codes_o, scales_o), ("bf16 gate", M))
