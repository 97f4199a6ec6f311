"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Bit-exact for scales, codes, planes and dequantized
weights; Y within 2e-3 (see gpu_util.assert_y_close)."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from oracle import fp6_oracle as O
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, from_np16, oracle_reference, to_np16
from layout_ref import pack_planes

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _quant(W):
    hi, lo, sc = P.fp6_quantize_pack(W)
    torch.cuda.synchronize()
    return hi, lo, sc


def _check_quant_bit_exact(Wnp16: np.ndarray):
    """quantize on the GPU and compare scales / codes / planes / W_hat with the oracle."""
    N, K = Wnp16.shape
    W = from_np16(Wnp16)
    hi, lo, sc = _quant(W)
    codes_o, scales_o = O.quantize(Wnp16)
    assert np.array_equal(to_np16(sc), scales_o)
    codes_g = P.fp6_unpack_codes(hi, lo, N, K).cpu().numpy()
    assert np.array_equal(codes_g, codes_o)
    hi_o, lo_o = pack_planes(codes_o)
    assert np.array_equal(hi.cpu().numpy(), hi_o)
    assert np.array_equal(lo.cpu().numpy(), lo_o)
    what_g = to_np16(P.fp6_dequantize(hi, lo, sc, N, K))
    assert np.array_equal(what_g, O.dequantize(codes_o, scales_o))
    return hi, lo, sc, codes_o, scales_o


# ------------------------------------------------------------------ offline step

def test_quantize_pack_config1_bit_exact():
    W = inputs.workload_weight("cfg1_single", 0, device=DEV)
    _check_quant_bit_exact(to_np16(W))


def test_quantize_pack_outlier_weights_bit_exact():
    W = inputs.weight(320, 704, seed=11, sigma=0.02, outlier_frac=0.001, device=DEV)
    _check_quant_bit_exact(to_np16(W))


def test_quantize_special_rows_bit_exact():
    rng = np.random.default_rng(4)
    N, K = 64, 128
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0] = 0                                                   # all-zero row, +0
    W[1] = np.float16(-0.0)                                    # all -0
    W[2] = 0; W[2, 5] = np.float16(6e-8); W[2, 6] = -np.float16(6e-8)   # amax/28 rounds to zero
    W[3] = (rng.standard_normal(K) * 1e-6).astype(np.float16)  # subnormal weights, subnormal scale
    W[4] = (rng.standard_normal(K) * 2000).astype(np.float16)  # large weights, S > 1
    mags = np.array([O.e3m2_value(c) for c in range(32)])
    mids = (mags[:-1] + mags[1:]) / 2
    for r, S0 in [(5, 2.0 ** -8), (6, 2.0 ** -2), (7, 2.0 ** -13)]:        # exact ties, both signs
        row = np.zeros(K)
        row[0] = 28 * S0
        row[1:32] = mids * S0
        row[33:64] = -mids * S0
        row[64:96] = mags * S0
        row[96:128] = -mags * S0
        W[r] = row.astype(np.float16)
        assert np.array_equal(W[r].astype(np.float64), row)
    W[8] = 0; W[8, 0] = np.float16(65504); W[8, 1] = np.float16(-65504); W[8, 2] = np.float16(30000)  # overflow of S*28
    W[9] = np.float16(0.3335); W[9, 3] = np.float16(0.01)     # |w|/S slightly above 28: saturation
    _check_quant_bit_exact(W.view(np.uint16))


def test_quantize_every_finite_fp16_value_at_many_scales():
    allw = np.arange(0, 0x7C00, dtype=np.uint16)
    rng = np.random.default_rng(6)
    amax_bits = [0x3C00, 0x2E66, 0x2C00, 0x3555, 0x0155, 0x0400, 0x7BFF, 0x1234, 0x0003, 0x5640] + \
        rng.integers(0x0400, 0x7BFF, 54).tolist()
    K = 63488 + 64 - 63488 % 64          # both signs of every finite value fit in one row
    rows = np.zeros((64, K), np.uint16)
    for r, ab in enumerate(amax_bits):
        w = allw[allw <= ab]
        row = np.concatenate([w, w | 0x8000])
        rows[r, :row.size] = row
        rows[r, row.size:] = ab
    _check_quant_bit_exact(rows)


# ------------------------------------------------------------------ planes

def test_unpack_is_inverse_of_documented_layout():
    rng = np.random.default_rng(8)
    N, K = 192, 320
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    hi, lo = pack_planes(codes)
    got = P.fp6_unpack_codes(torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), N, K)
    assert np.array_equal(got.cpu().numpy(), codes)
    for c in range(64):
        same = np.full((64, 64), c, np.uint8)
        hi, lo = pack_planes(same)
        got = P.fp6_unpack_codes(torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), 64, 64)
        assert np.array_equal(got.cpu().numpy(), same), c


def test_quantize_of_dequantized_is_identity_on_gpu():
    # rows hold S0 * value(c) for all 64 codes (incl. -0): quantize must return the codes,
    # and dequantize must return the same fp16 bits
    S0 = 2.0 ** -7
    vals = np.array([abs(O.e3m2_value(c)) for c in range(64)]) * S0
    bits = vals.astype(np.float16).view(np.uint16) | np.array([(c >> 5) << 15 for c in range(64)], np.uint16)
    W = np.tile(bits, (64, 1))
    hi, lo, sc = _quant(from_np16(W))
    assert np.array_equal(P.fp6_unpack_codes(hi, lo, 64, 64).cpu().numpy(), np.tile(np.arange(64, dtype=np.uint8), (64, 1)))
    assert np.array_equal(to_np16(P.fp6_dequantize(hi, lo, sc, 64, 64)), W)


# ------------------------------------------------------------------ hot path

NO_BS = P.binding.FP6_HINT_DEQUANT(1)     # ablation: integer exponent arithmetic instead of the bias shift
HMUL = P.binding.FP6_HINT_DEQUANT(2)      # ablation: fp16 multiply by 2^12
VARIANTS = [(P.FP6_VARIANT_DECODE, 1), (P.FP6_VARIANT_DECODE, 2), (P.FP6_VARIANT_GEMM, 1), (P.FP6_VARIANT_GEMM, 2),
            (P.FP6_VARIANT_DECODE | NO_BS, 1), (P.FP6_VARIANT_DECODE | NO_BS, 4), (P.FP6_VARIANT_GEMM | NO_BS, 1),
            (P.FP6_VARIANT_GEMM | NO_BS, 2), (P.FP6_VARIANT_DECODE | HMUL, 2), (P.FP6_VARIANT_GEMM | HMUL, 1)]


@pytest.mark.parametrize("variant,split", VARIANTS)
def test_one_hot_rows_read_back_dequantized_weights_bit_exact(variant, split):
    # X = one-hot rows: Y[m, n] must be RNE_fp16(S_n * value(code[n, k_m])) exactly - through
    # the MFMA path, FP6 subnormals (fp16 subnormal operands after the bias shift) included
    N, K = 128, 256
    rng = np.random.default_rng(12)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    codes[:, :64] = np.arange(64, dtype=np.uint8)[None, :]          # every code, every row
    hi, lo = pack_planes(codes)
    scales = np.linspace(0.004, 0.05, N).astype(np.float16).view(np.uint16)
    what = O.dequantize(codes, scales)
    hi_d, lo_d, sc_d = torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), from_np16(scales)
    ks = list(range(0, 64)) + [100, 255, 128, 191] + list(range(64, 76))
    # a sum that starts at +0 cannot return -0: zero weights compare without their sign
    what_cmp = np.where((what & 0x7FFF) == 0, 0, what).astype(np.uint16)
    for k0 in range(0, len(ks), 16):
        cols = ks[k0:k0 + 16]
        X = torch.zeros((len(cols), K), dtype=torch.float16, device=DEV)
        for m, k in enumerate(cols):
            X[m, k] = 1.0
        if variant & 0xFF == P.FP6_VARIANT_GEMM:
            X = torch.cat([X, X, X[:1]])                           # M = 33: ragged
        Y = P.fp6_linear_variant(X, hi_d, lo_d, sc_d, N, K, variant, split)
        torch.cuda.synchronize()
        Yb = to_np16(Y)
        Yb = np.where((Yb & 0x7FFF) == 0, 0, Yb).astype(np.uint16)
        for m, k in enumerate(cols):
            assert np.array_equal(Yb[m], what_cmp[:, k]), (m, k)


@pytest.mark.parametrize("M", [1, 3, 16])
@pytest.mark.parametrize("split", [1, 2, 4])
def test_decode_tiny_shapes_vs_bruteforce_oracle(M, split):
    N, K = 256, 256
    W = inputs.weight(N, K, seed=100 + M, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=200 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE, split)
    assert_y_close(Y, Yref, (M, split))


@pytest.mark.parametrize("M", [1, 17, 33, 64, 100, 129, 300])
@pytest.mark.parametrize("split", [1, 2])
def test_gemm_shapes_vs_oracle(M, split):
    N, K = 320, 512           # N not a multiple of 256: the last workgroup has idle wavefronts
    W = inputs.weight(N, K, seed=300 + M, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=400 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_GEMM, split)
    assert_y_close(Y, Yref, (M, split))


def test_config1_full_matrix():
    W = inputs.workload_weight("cfg1_single", 0, device=DEV)
    X = inputs.activation(1, 1024, seed=inputs.workload_seed("cfg1_single", 900), device=DEV)
    hi, lo, sc, codes_o, scales_o = _check_quant_bit_exact(to_np16(W))
    Yref = O.linear(to_np16(X), codes_o, scales_o)
    Y = P.fp6_linear(X, hi, lo, sc, 1024, 1024)
    assert_y_close(Y, Yref, "cfg1")


def test_constant_code_closed_form():
    # all codes = c, X = ones: Y = S * value(c) * K exactly representable
    N, K = 64, 256
    for c in [1, 12, 31, 45, 63]:
        hi, lo = pack_planes(np.full((N, K), c, np.uint8))
        sc = torch.full((N,), 2.0 ** -6, dtype=torch.float16, device=DEV)
        X = torch.ones((2, K), dtype=torch.float16, device=DEV)
        for variant in (P.FP6_VARIANT_DECODE, P.FP6_VARIANT_GEMM):
            Y = P.fp6_linear_variant(X, torch.from_numpy(hi).to(DEV), torch.from_numpy(lo).to(DEV), sc, N, K, variant, 1)
            assert torch.all(Y.double() == 2.0 ** -6 * O.e3m2_value(c) * K), (c, variant)


@pytest.mark.parametrize("M", [1, 2, 4, 5, 16])
@pytest.mark.parametrize("split", [2, 3, 4, 6, 8, 12, 24])
@pytest.mark.parametrize("meet", [1, 2])
def test_decode_slices_meet_at_counter_or_pairwise(M, split, meet):
    # both ways of adding K-slices, split counts that are not powers of two (tree nodes with a
    # single child), one workspace shared by every call and left zero by each
    N, K = 192, 64 * 24
    B = P.binding
    W = inputs.weight(N, K, seed=700 + split, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=710 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    variant = P.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(meet)
    ws = P.new_workspace(P.fp6_linear_variant_workspace_bytes(M, N, K, P.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(1), split), DEV)
    Ya = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    assert_y_close(Ya, Yref, (M, split, meet))
    # the other protocol on the same workspace, then this one again: bit-identical, zero region clean
    P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(3 - meet), split, workspace=ws)
    Yb = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Ya, Yb)
    assert torch.count_nonzero(ws[:B.FP6_WORKSPACE_ZERO_BYTES]).item() == 0


@pytest.mark.parametrize("M", [1, 16, 40, 100, 300])
@pytest.mark.parametrize("ablation", [NO_BS, HMUL])
def test_no_bias_shift_ablation_matches_oracle_and_the_bias_shift_path(M, ablation):
    # Section 5.2 ablation: same numbers by run-time exponent arithmetic.  Every product and the
    # scale multiply are the same real numbers times an exact power of two, so with the same
    # summation order the two paths agree bit for bit.
    N, K = 640, 1024
    W = inputs.weight(N, K, seed=900 + M, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=910 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    fam = P.FP6_VARIANT_DECODE if M <= 16 else P.FP6_VARIANT_GEMM
    Ya = P.fp6_linear_variant(X, hi, lo, sc, N, K, fam | ablation, 1)
    Yb = P.fp6_linear_variant(X, hi, lo, sc, N, K, fam, 1)
    assert_y_close(Ya, Yref, (M, "ablation"))
    assert torch.equal(Ya, Yb)


@pytest.mark.parametrize("M", [1, 3, 16])
@pytest.mark.parametrize("split,meet", [(1, 0), (2, 0), (2, 1), (4, 0), (4, 2), (6, 1)])
@pytest.mark.parametrize("depth", [0, 8])
def test_decode_half_tile_workgroups(M, split, meet, depth):
    # workgroups that own 32 channels: same results as the oracle, whatever the way the K-slices meet
    N, K = 320, 64 * 24
    B = P.binding
    W = inputs.weight(N, K, seed=800 + split, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=810 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    variant = P.FP6_VARIANT_DECODE | B.FP6_HINT_HALF(1) | B.FP6_HINT_MEET(meet) | B.FP6_HINT_DEPTH(depth)
    ws = P.new_workspace(P.fp6_linear_variant_workspace_bytes(M, N, K, P.FP6_VARIANT_DECODE | B.FP6_HINT_MEET(1), max(split, 2)), DEV)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    assert_y_close(Y, Yref, (M, split, meet))
    Y2 = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)
    assert torch.count_nonzero(ws[:B.FP6_WORKSPACE_ZERO_BYTES]).item() == 0


@pytest.mark.parametrize("width", [8, 4])
@pytest.mark.parametrize("M,bm,split", [(20, 32, 1), (33, 32, 3), (70, 64, 2), (64, 64, 1), (130, 128, 2), (300, 128, 1)])
def test_tiled_kernel_workgroup_widths(width, M, bm, split):
    # workgroups of 8 or 4 wavefronts (512 or 256 output channels); N = 11 channel blocks, so the last
    # workgroup of either width is ragged
    N, K = 704, 64 * 12
    B = P.binding
    W = inputs.weight(N, K, seed=1700 + width, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=1710 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    variant = P.FP6_VARIANT_GEMM | B.FP6_HINT_WIDTH(width) | B.FP6_HINT_BLOCK_M(bm)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split)
    torch.cuda.synchronize()
    assert_y_close(Y, Yref, (width, M, bm, split))


@pytest.mark.parametrize("M,N,K,split", [(100, 320, 1024, 1), (130, 256, 2048, 2), (300, 704, 1536, 4), (512, 1024, 768, 1),
                                         (129, 64, 128, 1), (512, 512, 4096, 8)])
def test_tiled_kernel_with_two_k_ways_inside_the_workgroup(M, N, K, split):
    """Eight wavefronts on a 128 x 256 block: two sets that take alternate k tiles and add their sums in LDS."""
    W = inputs.weight(N, K, seed=210 + M, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=211 + split, device=DEV)
    hi, lo, sc = _quant(W)
    variant = (P.FP6_VARIANT_GEMM | P.binding.FP6_HINT_BLOCK_M(128) | P.binding.FP6_HINT_WIDTH(4) |
               P.binding.FP6_HINT_KWAYS(2))
    plan = P.fp6_linear_plan(M, N, K, variant=variant, split_k=split)
    assert (plan["waves"], plan["width"], plan["block_m"], plan["split_k"]) == (8, 4, 128, split)
    ws = P.new_workspace(max(plan["workspace_bytes"], 16), DEV)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    Y2 = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split, workspace=ws)
    torch.cuda.synchronize()
    _, _, Yref = oracle_reference(W, X)
    assert_y_close(Y, Yref, "two K-ways, split %d" % split)
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16)), "not reproducible"
    if plan["workspace_bytes"]:
        assert not ws[:min(plan["workspace_bytes"], P.binding.FP6_WORKSPACE_ZERO_BYTES)].any()


def test_two_k_ways_need_an_even_number_of_k_tiles_per_slice_and_the_128_by_256_block():
    B = P.binding
    kw = P.FP6_VARIANT_GEMM | B.FP6_HINT_KWAYS(2)
    a = torch.zeros(64, dtype=torch.uint8, device=DEV)
    L, st = B.lib(), torch.cuda.current_stream().cuda_stream
    def rc(M, N, K, variant, split):
        return L.fp6_linear_variant(a.data_ptr(), M, a.data_ptr(), a.data_ptr(), a.data_ptr(), N, K, a.data_ptr(), None, 0, st,
                                    variant, split)
    assert rc(128, 256, 192, kw | B.FP6_HINT_BLOCK_M(128) | B.FP6_HINT_WIDTH(4), 1) == -5       # three k tiles
    assert rc(128, 256, 384, kw | B.FP6_HINT_BLOCK_M(128) | B.FP6_HINT_WIDTH(4), 2) == -5       # two slices of three
    assert rc(128, 256, 512, kw | B.FP6_HINT_BLOCK_M(64) | B.FP6_HINT_WIDTH(4), 1) == -5
    assert rc(128, 256, 512, kw | B.FP6_HINT_BLOCK_M(128) | B.FP6_HINT_WIDTH(8), 1) == -5
    assert rc(8, 256, 512, P.FP6_VARIANT_DECODE | B.FP6_HINT_KWAYS(2), 1) == -5


@pytest.mark.parametrize("M", [17, 24, 32, 33, 47, 48, 64])
@pytest.mark.parametrize("split", [1, 2, 6])
def test_decode_family_with_several_row_blocks(M, split):
    # the streaming kernel with two or four blocks of 16 rows of X per wavefront (M <= 64)
    N, K = 192, 64 * 24
    W = inputs.weight(N, K, seed=1800 + split, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=1810 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    ws = P.new_workspace(P.fp6_linear_variant_workspace_bytes(M, N, K, P.FP6_VARIANT_DECODE, split), DEV)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE, split, out=out, workspace=ws)
    assert_y_close(Y, Yref, (M, split))
    Y2 = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE, split, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)


def test_split_and_unsplit_agree_and_workspace_is_reusable():
    N, K, M = 512, 2048, 8
    W = inputs.weight(N, K, seed=31, sigma=0.02, outlier_frac=0.001, device=DEV)
    hi, lo, sc = _quant(W)
    ws = P.new_workspace(P.fp6_linear_variant_workspace_bytes(M, N, K, P.FP6_VARIANT_DECODE, 8), DEV)
    ys = []
    for it in range(6):
        X = inputs.activation(M, K, seed=500 + it, device=DEV)
        Y1 = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE, 1)
        Y8 = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE, 8, workspace=ws)
        Y8b = P.fp6_linear_variant(X, hi, lo, sc, N, K, P.FP6_VARIANT_DECODE, 8, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(Y8, Y8b)                       # deterministic, counters were reset
        # split and unsplit differ only by fp32 summation order: within one fp16 ulp-ish
        d = (Y1.float() - Y8.float()).abs().max().item()
        assert d <= 2e-3 * Y1.float().abs().max().item()
        ys.append(Y8)
    assert torch.count_nonzero(ws[:P.binding.FP6_WORKSPACE_ZERO_BYTES]).item() == 0
    assert not torch.equal(ys[0], ys[1])


def test_linearity():
    N, K, M = 256, 1024, 16
    W = inputs.weight(N, K, seed=41, device=DEV)
    hi, lo, sc = _quant(W)
    X1 = inputs.activation(M, K, seed=42, device=DEV)
    X2 = inputs.activation(M, K, seed=43, device=DEV)
    Ya = P.fp6_linear(X1, hi, lo, sc, N, K).float() + P.fp6_linear(X2, hi, lo, sc, N, K).float()
    Yb = P.fp6_linear((X1.float() + X2.float()).half(), hi, lo, sc, N, K).float()
    assert (Ya - Yb).abs().max().item() <= 4e-3 * Yb.abs().max().item()


@pytest.mark.parametrize("M", [1, 4, 16, 32, 128])
def test_llama7b_qkvo_full_matrix(M):
    N = K = 4096
    W = inputs.workload_weight("cfg2_llama7b", 0, device=DEV)
    X = inputs.activation(M, K, seed=inputs.workload_seed("cfg2_llama7b", 900 + M), device=DEV)
    hi, lo, sc = _quant(W)
    codes_o, scales_o, Yref = oracle_reference(W, X)
    assert np.array_equal(to_np16(sc), scales_o)
    assert np.array_equal(P.fp6_unpack_codes(hi, lo, N, K).cpu().numpy(), codes_o)
    Y = P.fp6_linear(X, hi, lo, sc, N, K)
    assert_y_close(Y, Yref, M)


# ------------------------------------------------------------------ extreme aspect ratios, degenerate inputs

@pytest.mark.parametrize("M,N,K", [(1, 65536, 64), (2, 64, 65536), (16, 64, 64), (2048, 128, 256), (1000, 64, 4096),
                                   (5, 128, 28672), (1, 24576, 128), (700, 1024, 64)])
def test_extreme_shapes_vs_oracle(M, N, K):
    # one tile in one direction and thousands in the other; many row blocks of X; a single tile
    W = inputs.weight(N, K, seed=2000 + N % 97 + K % 89, sigma=0.02, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=2100 + M, device=DEV)
    hi, lo, sc = _quant(W)
    _, _, Yref = oracle_reference(W, X)
    Y = P.fp6_linear(X, hi, lo, sc, N, K)
    torch.cuda.synchronize()
    assert_y_close(Y, Yref, (M, N, K))


@pytest.mark.parametrize("M", [1, 16, 64])
def test_all_zero_weights_and_zero_rows_give_exact_zeros(M):
    N, K = 256, 512
    W = inputs.weight(N, K, seed=5, device=DEV)
    W[::2] = 0                                   # every other output channel: S = 0
    X = inputs.activation(M, K, seed=6, device=DEV)
    hi, lo, sc = _quant(W)
    Y = P.fp6_linear(X, hi, lo, sc, N, K)
    torch.cuda.synchronize()
    assert torch.isfinite(Y).all()
    assert torch.count_nonzero(Y[:, ::2]).item() == 0
    assert torch.count_nonzero(Y[:, 1::2]).item() > 0
    W[:] = 0
    hi, lo, sc = _quant(W)
    assert torch.count_nonzero(P.fp6_linear(X, hi, lo, sc, N, K)).item() == 0


def test_zero_activations_give_zeros_and_results_do_not_depend_on_stale_output():
    N, K, M = 192, 384, 9
    W = inputs.weight(N, K, seed=7, device=DEV)
    hi, lo, sc = _quant(W)
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    P.fp6_linear(torch.zeros((M, K), dtype=torch.float16, device=DEV), hi, lo, sc, N, K, out=out)
    torch.cuda.synchronize()
    assert torch.count_nonzero(out).item() == 0          # every element written, none left NaN


@pytest.mark.parametrize("variant,split", [(1, 1), (1, 2), (1, 4), (2, 1), (2, 2)])
def test_overflow_and_non_finite_activations_propagate_as_in_the_oracle(variant, split):
    """Nothing is clamped or detected: results beyond the fp16 range become infinities of the right sign, an infinite
    activation gives +-inf (NaN where it meets a zero weight or an opposite infinity), a NaN poisons its row, and the
    other rows are untouched - through the streaming and the tiled kernel, with and without a K-split (two slices of
    the streaming kernel meet pairwise, four at a counter)."""
    N, K, M = 256, 512, 6
    W = inputs.weight(N, K, seed=5100, sigma=0.05, outlier_frac=0.001, device=DEV)
    X = inputs.activation(M, K, seed=5101, device=DEV)
    X[1, :] = 60000.0
    X[2, 5] = float("inf")
    X[3, 7] = float("nan")
    X[4, 300] = float("-inf")
    X[4, 301] = float("inf")
    hi, lo, sc = _quant(W)
    codes_o, scales_o = O.quantize(to_np16(W))
    with np.errstate(all="ignore"):
        Yref = O.linear(to_np16(X), codes_o, scales_o)
    Y = P.fp6_linear_variant(X, hi, lo, sc, N, K, variant, split)
    torch.cuda.synchronize()
    y = Y.cpu().to(torch.float64).numpy()
    # the oracle's result is not rounded to fp16: what lies beyond the largest fp16 number (65504; ties at 65520) must
    # come out infinite, what lies well inside must not; the narrow band between is left to either
    with np.errstate(invalid="ignore"):
        big, inside = np.abs(Yref) > 65600, np.abs(Yref) < 65400
    decided = big | inside | np.isnan(Yref)
    assert (big[1] & np.isfinite(Yref[1])).any() and inside[1].any(), "row 1 should straddle the fp16 range"
    assert np.isnan(Yref[3]).all() and not np.isfinite(Yref[2]).any()
    assert np.array_equal(np.isnan(y), np.isnan(Yref))
    assert np.array_equal(np.isposinf(y) & decided, big & (Yref > 0))
    assert np.array_equal(np.isneginf(y) & decided, big & (Yref < 0))
    assert_y_close(Y[[0, 5]], Yref[[0, 5]], (variant, split))
    # the finite part of the overflowing row: 2e-3 of the value plus one fp16 step at that size
    fin = inside[1]
    err = np.abs(y[1][fin] - Yref[1][fin])
    assert np.isfinite(y[1][fin]).all() and (err <= 2e-3 * np.abs(Yref[1][fin]) + 32.0).all()


def test_probe_kernels_run_and_reject_bad_arguments():
    """The measurement aids launch, write their sinks, and refuse sinks that are too small."""
    buf = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    buf[12345] ^= 0x5A5A5
    sink = torch.zeros(64 * 4, dtype=torch.int32, device=DEV)
    P.fp6_probe_read(buf, 64, sink)
    torch.cuda.synchronize()
    # the fold of all words of the buffer: the xor of 0 .. 2^20 - 1 is 0, so the planted word is what is left
    total = 0
    for w in sink.cpu().numpy().tolist():
        total ^= w & 0xFFFFFFFF
    assert total == 0x5A5A5
    with pytest.raises(P.Fp6Error):
        P.fp6_probe_read(buf, 65, sink)
    out = torch.full((4 * 256,), float("nan"), dtype=torch.float32, device=DEV)
    flop = P.fp6_probe_mfma(4, 3, False, out)
    assert flop == 4 * 4 * 8 * 3 * 16384
    assert P.fp6_probe_mfma(4, 3, True, out, wide=True) == 2 * flop
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    P.fp6_probe_mfma(4, 3, False, out)
    torch.cuda.synchronize()
    assert (out == 0).all()                   # zero operands
    with pytest.raises(P.Fp6Error):
        P.fp6_probe_mfma(5, 3, False, out)
    # the form with integer instructions between the MFMAs does the same MFMAs: same sums, plus a parity bit
    plain = torch.empty_like(out)
    P.fp6_probe_mfma(4, 3, True, plain)
    assert P.fp6_probe_mfma(4, 3, True, out, valu_mix=True) == flop
    torch.cuda.synchronize()
    extra = (out.double() - plain.double()).abs()
    tol = 1e-5 * (1 + plain.abs().max().item())          # the bit is added in fp32
    assert ((extra <= tol) | ((extra - 1).abs() <= tol)).all() and torch.isfinite(out).all()


@pytest.mark.parametrize("seed", range(4))
def test_automatic_plans_on_random_shapes(seed):
    """Whatever kernel, workgroup shape and K-split the planner picks: sampled channels against the oracle.
    Shapes are log-uniform in N, K <= 8192 and M <= 700, eight per seed."""
    import math
    rng = np.random.default_rng(4200 + seed)
    for i in range(8):
        N = 64 * int(round(math.exp(rng.uniform(0.0, math.log(128)))))
        K = 64 * int(round(math.exp(rng.uniform(0.0, math.log(128)))))
        M = int(round(math.exp(rng.uniform(0.0, math.log(700)))))
        W = inputs.weight(N, K, seed=4300 + 10 * seed + i, sigma=0.02, outlier_frac=0.001, device=DEV)
        X = inputs.activation(M, K, seed=4400 + 10 * seed + i, device=DEV)
        rows = np.unique(np.concatenate([[0, N - 1], rng.choice(N, size=min(N, 32), replace=False)]))
        ridx = torch.from_numpy(rows).to(DEV)
        codes_o, scales_o = O.quantize(to_np16(W[ridx]))
        hi, lo, sc = _quant(W)
        Y = P.fp6_linear(X, hi, lo, sc, N, K)
        torch.cuda.synchronize()
        assert np.array_equal(to_np16(sc[ridx]), scales_o), (M, N, K)
        assert_y_close(Y[:, ridx], O.linear(to_np16(X), codes_o, scales_o), (M, N, K))


@pytest.mark.parametrize("seed", range(3))
def test_automatic_plans_on_random_prefill_shapes(seed):
    """The same for prefill sizes: 65 <= M < 700 rows, N up to 12.7 K and K up to 16.6 K, uniform, eight per seed -
    the region of the 128-row blocks, with and without a K-split or two K-ways inside the workgroup."""
    rng = np.random.default_rng(4700 + seed)
    for i in range(8):
        N = 64 * int(rng.integers(16, 200))
        K = 64 * int(rng.integers(16, 260))
        M = int(rng.integers(65, 700))
        W = inputs.weight(N, K, seed=4800 + 10 * seed + i, sigma=0.02, outlier_frac=0.001, device=DEV)
        X = inputs.activation(M, K, seed=4900 + 10 * seed + i, device=DEV)
        rows = np.unique(np.concatenate([[0, N - 1], rng.choice(N, size=24, replace=False)]))
        ridx = torch.from_numpy(rows).to(DEV)
        codes_o, scales_o = O.quantize(to_np16(W[ridx]))
        hi, lo, sc = _quant(W)
        Y = P.fp6_linear(X, hi, lo, sc, N, K)
        torch.cuda.synchronize()
        text = P.plan_text(P.fp6_linear_plan(M, N, K))
        assert np.array_equal(to_np16(sc[ridx]), scales_o), (M, N, K, text)
        assert_y_close(Y[:, ridx], O.linear(to_np16(X), codes_o, scales_o), (M, N, K, text))
