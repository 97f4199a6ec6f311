"""Pins for the CPU oracle: everything here checks oracle/ against facts fixed by the
paper or by mathematics (closed forms, a library's fp16 arithmetic, exact rational
brute force, invariants) - never against the oracle's own formulas and never against
the HIP path."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import fp6_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e3m2_magnitudes.txt")


def golden_magnitudes():
    mags = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        mags[int(f[0])] = (f[1], f[2], float(f[3]))
    return mags


# ------------------------------------------------------------------ value set

def test_e3m2_values_match_paper_worked_table():
    mags = golden_magnitudes()
    assert sorted(mags) == list(range(32))
    for c5, (eee, mm, val) in mags.items():
        assert c5 == int(eee + mm, 2)
        assert O.e3m2_value(c5) == val
        assert O.e3m2_value(c5 | 32) == -val


def test_e3m2_facts_fixed_by_the_text():
    vals = [O.e3m2_value(c) for c in range(64)]
    # Section 4: max/min achievable value is +-28 = +-1 * 2^4 * 1.75
    assert max(vals) == 28.0 == 2.0 ** 4 * 1.75 and min(vals) == -28.0
    assert vals[0b011111] == 28.0 and vals[0b111111] == -28.0
    # no NaN / inf codes (Section 4 footnote)
    assert all(np.isfinite(v) for v in vals)
    # bias 3 (Section 5.2): exponent field 3, mantissa 0 is 1.0
    assert vals[0b001100] == 1.0
    # subnormals: exponent field 0, zero included (Section 5.2 footnote); 4 per sign
    assert [vals[c] for c in range(4)] == [0.0, 1 / 16, 2 / 16, 3 / 16]
    # smallest normal 2^(1-3)
    assert vals[0b000100] == 0.25
    # strictly increasing magnitudes in the 5-bit code; sign symmetry; -0 exists
    assert all(vals[c + 1] > vals[c] for c in range(31))
    assert all(vals[c | 32] == -vals[c] for c in range(32))
    assert np.signbit(vals[32]) and vals[32] == 0.0


def test_e3m2_closed_form_eq2():
    # Eq. 2 with e = 3, b = 3: normal x = (-1)^s 2^(E-3) (1 + m/4); subnormal 2^(1-3) (m/4)
    for c in range(64):
        s, E, m = c >> 5, (c >> 2) & 7, c & 3
        x = Fraction(2) ** (E - 3) * (1 + Fraction(m, 4)) if E else Fraction(1, 4) * Fraction(m, 4)
        assert Fraction(O.e3m2_value(c)) == (-x if s else x)


def test_bias_shift_identity_eq5_numpy_fp16():
    # Eq. 5: the 6 bits read with bias 15 are an fp16 whose value * 2^12 is the FP6 value;
    # decoded here by numpy's float16, not by the oracle.
    for c in range(64):
        h = np.array([O.bias_shift_bits(c)], np.uint16).view(np.float16)[0]
        assert float(h) * 4096.0 == O.e3m2_value(c)
        assert np.signbit(h) == bool(c & 32)
    # subnormal FP6 codes must be subnormal fp16 patterns (exponent field stays zero)
    for c in list(range(4)) + list(range(32, 36)):
        assert (O.bias_shift_bits(c) >> 10) & 0x1F == 0
    # pure padding: only bits 15 and 12..8 may ever be set
    assert all(O.bias_shift_bits(c) & ~0x9F00 == 0 for c in range(64))


def test_bias_shift_identity_torch_e5m2():
    # an 8-bit float with 5 exponent bits (bias 15) and 2 mantissa bits is the top byte of
    # fp16: the byte s00eeemm read by torch as float8_e5m2 must be value * 2^-12.
    b = torch.tensor([O.bias_shift_bits(c) >> 8 for c in range(64)], dtype=torch.uint8)
    v = b.view(torch.float8_e5m2).to(torch.float32) * 4096.0
    assert v.tolist() == [O.e3m2_value(c) for c in range(64)]


# ------------------------------------------------------------------ fp16 helpers

def test_half_to_double_all_patterns_vs_numpy():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([O.half_to_double(int(b)) for b in bits])
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.array_equal(np.signbit(got[fin]), np.signbit(ref[fin]))
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))


def test_round_helper_vs_numpy_rne():
    rng = np.random.default_rng(1)
    # exact doubles (num / 2^24 with den = 1): numpy rounds a double to fp16 with RNE
    nums = np.concatenate([rng.integers(0, 1 << 41, 20000), rng.integers(0, 1 << 13, 5000),
                           np.arange(0, 5000)])
    for n in nums:
        ref = np.array([float(n) / 2 ** 24]).astype(np.float16).view(np.uint16)[0]
        assert O.round_ratio_to_half(int(n), 1) == int(ref), n
    # all fp16 midpoints (ties) and their neighbours, den = 2 gives half-units
    for b in list(range(0, 0x7BFF, 37)) + [0, 1, 2, 1022, 1023, 1024, 0x7BFE, 0x7BFF]:
        lo = Fraction(float(np.array([b], np.uint16).view(np.float16)[0]))
        hi = Fraction(float(np.array([b + 1], np.uint16).view(np.float16)[0])) if b + 1 < 0x7C00 else Fraction(65536)
        mid = (lo + hi) / 2
        num = mid * 2 ** 25
        assert num.denominator == 1
        want = b if b % 2 == 0 else b + 1      # ties to even significand (overflow: inf = 0x7C00)
        assert O.round_ratio_to_half(int(num), 2) == want
        assert O.round_ratio_to_half(int(num) - 1, 2) == b
        assert O.round_ratio_to_half(int(num) + 1, 2) == b + 1


# ------------------------------------------------------------------ scale

def _nearest_half_exact(x: Fraction) -> int:
    """bits of the fp16 nearest to x >= 0 (ties to even), by exact search around numpy's guess."""
    guess = int(np.array([float(x)]).astype(np.float16).view(np.uint16)[0])
    best = None
    for b in range(max(0, guess - 2), min(0x7BFF, guess + 2) + 1):
        v = Fraction(float(np.array([b], np.uint16).view(np.float16)[0]))
        d = abs(v - x)
        if best is None or d < best[0] or (d == best[0] and b % 2 == 0 and best[1] % 2 == 1):
            best = (d, b)
    return best[1]


def test_scale_is_amax_over_28_rounded_once_every_fp16_amax():
    # every positive finite fp16 as the row maximum (31743 cases), exact rational check
    for b in range(1, 0x7C00):
        amax = Fraction(float(np.array([b], np.uint16).view(np.float16)[0]))
        row = np.array([0, b, b | 0x8000 if b % 2 else 0], np.uint16)
        assert O.row_scale(row) == _nearest_half_exact(amax / 28), b


def test_scale_special_rows():
    assert O.row_scale(np.zeros(8, np.uint16)) == 0                       # all-zero row
    assert O.row_scale(np.array([0x8000, 0], np.uint16)) == 0             # -0
    # negative maximum counts by magnitude
    r = np.array([1.0, -7.0, 3.0], np.float16)
    assert np.array([O.row_scale(r)], np.uint16).view(np.float16)[0] == np.float16(0.25)
    # rows built as S0 * value(code) with 28*S0 representable return S0 exactly
    for S0 in [2.0 ** -10, 2.0 ** -3, 1.0, 0.013671875, 3.0 * 2.0 ** -12, 2.0 ** -20]:
        row = np.array([S0 * O.e3m2_value(c) for c in range(64)], np.float64).astype(np.float16)
        assert float(row.max()) == 28 * S0
        assert np.array([O.row_scale(row)], np.uint16).view(np.float16)[0] == np.float16(S0)
    with pytest.raises(ValueError):
        O.row_scale(np.array([1.0, np.inf], np.float16))
    with pytest.raises(ValueError):
        O.row_scale(np.array([np.nan, 1.0], np.float16))


# ------------------------------------------------------------------ codes

MAGS = [v for (_, _, v) in (golden_magnitudes()[c] for c in range(32))]


def _brute_code(w16: np.float16, S16: np.float16) -> int:
    """exact rational argmin over the paper's 32 magnitudes, ties to the even code."""
    s = 32 if np.signbit(w16) else 0
    S = Fraction(float(S16))
    if S == 0:
        return s
    q = abs(Fraction(float(w16))) / S
    d = [abs(q - Fraction(m)) for m in MAGS]
    best = min(d)
    cands = [i for i in range(32) if d[i] == best]
    pick = cands[0] if len(cands) == 1 else [i for i in cands if i % 2 == 0][0]
    return s | pick


def test_codes_bruteforce_random_rows():
    rng = np.random.default_rng(7)
    for trial in range(6):
        sigma = [0.02, 0.015, 1.0, 30.0, 1e-4, 0.02][trial]
        W = (rng.standard_normal((4, 160)) * sigma)
        if trial in (0, 1):
            W[rng.random(W.shape) < 0.02] *= 10
        W = W.astype(np.float16)
        codes, scales = O.quantize(W)
        S = scales.view(np.float16)
        for n in range(W.shape[0]):
            assert scales[n] == _nearest_half_exact(Fraction(float(np.abs(W[n]).max())) / 28)
            for k in range(W.shape[1]):
                assert codes[n, k] == _brute_code(W[n, k], S[n]), (trial, n, k)


def test_codes_exact_ties_go_to_even_code():
    # w = midpoint * S exactly, S a power of two, row max = 28 S
    for S0 in [2.0 ** -8, 2.0 ** -2]:
        mids = [(MAGS[i] + MAGS[i + 1]) / 2 for i in range(31)]
        row = np.array([28 * S0] + [m * S0 for m in mids] + [-m * S0 for m in mids], np.float64)
        row16 = row.astype(np.float16)
        assert np.array_equal(row16.astype(np.float64), row)        # all exactly representable
        codes, scales = O.quantize(row16[None, :])
        assert scales.view(np.float16)[0] == np.float16(S0)
        for i in range(31):
            even = i if i % 2 == 0 else i + 1
            assert codes[0, 1 + i] == even
            assert codes[0, 1 + 31 + i] == 32 | even
        # one fp16 ulp to either side of a midpoint goes to the nearer code
        for i in range(4, 31):
            m16 = np.float16(mids[i] * S0)
            below = np.nextafter(m16, np.float16(0))
            above = np.nextafter(m16, np.float16(np.inf))
            c, _ = O.quantize(np.array([[28 * S0, below, above]], np.float16))
            assert (c[0, 1], c[0, 2]) == (i, i + 1)


def test_quantize_is_idempotent_on_the_grid():
    # quantize(S0 * value(c)) == c for all 64 codes, -0 included
    for S0 in [2.0 ** -9, 0.013671875, 1.0, 2.0 ** -20]:
        row = np.array([S0 * abs(O.e3m2_value(c)) for c in range(64)], np.float64).astype(np.float16)
        bits = row.view(np.uint16) | np.array([(c >> 5) << 15 for c in range(64)], np.uint16)
        codes, scales = O.quantize(bits[None, :])
        assert codes[0].tolist() == list(range(64))
        # and dequantize returns the same bits: quantize(dequantize(c)) == c
        back, _ = O.quantize(O.dequantize(codes, scales))
        assert back[0].tolist() == list(range(64))


def test_quantize_invariants_on_workload_like_rows():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((8, 4096)) * 0.02
    W[rng.random(W.shape) < 0.001] *= 10
    W = W.astype(np.float16)
    codes, scales = O.quantize(W)
    S = scales.view(np.float16).astype(np.float64)
    vals = np.array([O.e3m2_value(c) for c in range(64)])
    q = vals[codes]
    Wd = W.astype(np.float64)
    for n in range(W.shape[0]):
        # the row's largest element decodes to +-28
        k = np.abs(Wd[n]).argmax()
        assert abs(q[n, k]) == 28.0 and np.sign(q[n, k]) == np.sign(Wd[n, k])
        # sign bit preserved everywhere
        assert np.array_equal(codes[n] >> 5, (W[n].view(np.uint16) >> 15).astype(np.uint8))
        # monotone: sorting w sorts the dequantized values
        order = np.argsort(Wd[n], kind="stable")
        assert np.all(np.diff(q[n, order]) >= 0)
        # error bound: half the local grid spacing (2 at the top binade; saturation adds at most S*28*2^-11)
        r = np.abs(Wd[n] / S[n])
        spacing = np.where(r < 0.25, 1 / 16, 2.0 ** (np.floor(np.log2(np.maximum(r, 0.25))) - 2))
        err = np.abs(Wd[n] / S[n] - q[n])
        assert np.all(err <= spacing / 2 + 28 * 2.0 ** -10)
    # saturation: |w|/S may exceed 28 slightly because S was rounded; it must still give 28
    row = np.array([0.3335, 0.3335, -0.3335, 0.01], np.float16)
    c, s = O.quantize(row[None, :])
    assert float(row[0]) / float(s.view(np.float16)[0]) > 28.0
    assert c[0, :3].tolist() == [31, 31, 63]


def test_zero_scale_rows_give_signed_zero_codes():
    row = np.array([0x0000, 0x8000, 0x0000, 0x8000], np.uint16)
    c, s = O.quantize(row[None, :])
    assert s[0] == 0 and c[0].tolist() == [0, 32, 0, 32]
    # amax so small that amax/28 rounds to zero
    row = np.array([0x0001, 0x8001, 0x000D, 0x0000], np.uint16)      # 13 * 2^-24 / 28 < 0.5 * 2^-24
    c, s = O.quantize(row[None, :])
    assert s[0] == 0 and c[0].tolist() == [0, 32, 0, 0]
    assert np.array_equal(O.dequantize(c, s)[0], np.array([0, 0x8000, 0, 0], np.uint16))
    Y = O.linear(np.ones((2, 4), np.float16), c, s)
    assert np.all(Y == 0)


# ------------------------------------------------------------------ 4+2 split

def test_split42_is_sign_exponent_plus_mantissa_and_round_trips():
    codes = np.arange(64, dtype=np.uint8)
    hi4, lo2 = O.split42(codes)
    for c in range(64):
        s, e, m = c >> 5, (c >> 2) & 7, c & 3
        assert hi4[c] == (s << 3 | e) and lo2[c] == m          # Section 5.1
    assert np.array_equal(O.join42(hi4, lo2), codes)
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 64, (37, 129), dtype=np.uint8)
    hi4, lo2 = O.split42(codes)
    assert hi4.max() < 16 and lo2.max() < 4
    assert np.array_equal(O.join42(hi4, lo2), codes)
    for c in range(64):
        same = np.full((3, 5), c, np.uint8)
        assert np.array_equal(O.join42(*O.split42(same)), same)


# ------------------------------------------------------------------ dequantize

def test_dequantize_vs_numpy_float_rounding():
    # W_hat = RNE_fp16(S * value(c)); numpy does the product in float64 (exact) and rounds once
    rng = np.random.default_rng(11)
    scales = np.concatenate([rng.integers(1, 0x7BFF, 300).astype(np.uint16),
                             np.array([0, 1, 2, 3, 0x03FF, 0x0400, 0x0401, 0x7BFF, 0x6892], np.uint16)])
    codes = np.tile(np.arange(64, dtype=np.uint8), (scales.size, 1))
    got = O.dequantize(codes, scales)
    vals = np.array([O.e3m2_value(c) for c in range(64)])
    with np.errstate(over="ignore"):
        ref = (scales.view(np.float16).astype(np.float64)[:, None] * vals[None, :]).astype(np.float16)
    assert np.array_equal(got, ref.view(np.uint16))
    # overflow case is IEEE: 0x6892 = 2340 = RNE(65504/28); 2340*28 = 65520 -> +inf
    assert got[-1, 31] == 0x7C00 and got[-1, 63] == 0xFC00


# ------------------------------------------------------------------ linear

def test_linear_bruteforce_fractions_tiny():
    rng = np.random.default_rng(5)
    M, N, K = 3, 4, 7
    X = rng.standard_normal((M, K)).astype(np.float16)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    scales = rng.integers(0x1000, 0x3C00, N).astype(np.uint16)
    Y = O.linear(X, codes, scales)
    for m in range(M):
        for n in range(N):
            S = Fraction(float(scales[n:n + 1].view(np.float16)[0]))
            acc = sum(Fraction(float(X[m, k])) * Fraction(MAGS[codes[n, k] & 31]) * (-1 if codes[n, k] & 32 else 1)
                      for k in range(K))
            exact = float(S * acc)
            assert abs(Y[m, n] - exact) <= 1e-13 * max(1.0, abs(exact))


def test_linear_equals_numpy_matmul_when_everything_is_exact():
    # small integers: every product and partial sum is exact in double, so the plain
    # definition must agree with numpy's float64 matmul to the last bit, in [M,N] layout
    rng = np.random.default_rng(9)
    M, N, K = 5, 6, 64
    X = rng.integers(-8, 9, (M, K)).astype(np.float16)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    scales = np.array([2.0 ** -k for k in range(N)], np.float16).view(np.uint16)
    Wv = np.array([[MAGS[c & 31] * (-1 if c & 32 else 1) for c in row] for row in codes])
    ref = (X.astype(np.float64) @ Wv.T) * scales.view(np.float16).astype(np.float64)[None, :]
    assert np.array_equal(O.linear(X, codes, scales), ref)
    # a transposed operand or swapped output layout would break this asymmetric case
    assert O.linear(X, codes, scales).shape == (M, N)


def test_linear_constant_code_closed_form():
    # all codes equal c, X all ones: Y = S * value(c) * K exactly
    K = 256
    for c in [1, 12, 31, 45, 63]:
        codes = np.full((2, K), c, np.uint8)
        scales = np.array([0.5, 0.125], np.float16).view(np.uint16)
        Y = O.linear(np.ones((1, K), np.float16), codes, scales)
        v = MAGS[c & 31] * (-1 if c & 32 else 1)
        assert Y.tolist() == [[0.5 * v * K, 0.125 * v * K]]


def test_linear_scale_applies_after_the_sum_and_uses_true_code_values():
    # Y must not round the dequantized weight to fp16 first: pick S and code whose product
    # is not an fp16 number and check the exact value survives
    S = np.array([0.0999755859375], np.float16)       # 11 significant bits
    codes = np.array([[23]], np.uint8)                # 7 = 1.75 * 4: product needs 13 bits
    Y = O.linear(np.array([[1.0]], np.float16), codes, S.view(np.uint16))
    assert Y[0, 0] == float(S[0]) * 7.0
    assert float(np.float16(Y[0, 0])) != Y[0, 0]


# ------------------------------------------------------------------ fine-grained (block-k) scales

def _rows(rng, N, K, sigma=0.02):
    W = (rng.standard_normal((N, K)) * sigma).astype(np.float16)
    W[rng.random((N, K)) < 0.002] *= np.float16(10.0)
    return W


def test_fgq_with_block_equal_to_row_is_the_row_wise_scheme():
    # Section 3: coarse-grained = block size equal to the row size
    rng = np.random.default_rng(21)
    W = _rows(rng, 6, 192)
    c1, s1 = O.quantize(W)
    c2, s2 = O.quantize_fgq(W, 192)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2[:, 0])
    X = rng.standard_normal((3, 192)).astype(np.float16)
    assert np.array_equal(O.linear(X, c1, s1), O.linear_fgq(X, c2, s2, 192))
    assert np.array_equal(O.dequantize(c1, s1), O.dequantize_fgq(c2, s2, 192))


def test_fgq_every_block_is_an_independent_row():
    # block-k quantization: every k elements have their own scale (Appendix A) - so quantizing
    # the [N, K] matrix in blocks equals quantizing the [N*K/block, block] matrix row-wise
    rng = np.random.default_rng(22)
    N, K = 5, 512
    W = _rows(rng, N, K)
    for block in (64, 128, 256):
        c, s = O.quantize_fgq(W, block)
        cr, sr = O.quantize(W.reshape(N * K // block, block))
        assert np.array_equal(c.reshape(-1, block), cr)
        assert np.array_equal(s.reshape(-1), sr)
        # each block's largest element sits on the largest code, and the scale is max/28 rounded once
        a = np.abs(W.astype(np.float64)).reshape(N, K // block, block)
        assert np.array_equal(s.view(np.float16), (a.max(axis=2) / 28.0).astype(np.float16))
        top = np.take_along_axis((c & 31).reshape(N, K // block, block), a.argmax(axis=2)[..., None], axis=2)
        assert np.all(top == 31)
        # finer blocks never quantize worse than coarser ones in the block's own max-norm bound
        err = np.abs(O.dequantize_fgq(c, s, block).view(np.float16).astype(np.float64) - W.astype(np.float64))
        bound = 2.0 * s.view(np.float16).astype(np.float64).repeat(block, axis=1) * (1 + 2.0 ** -10) + 2.0 ** -24
        assert np.all(err <= bound)


def test_fgq_dequantize_uses_the_scale_of_the_elements_own_block():
    codes = np.tile(np.arange(64, dtype=np.uint8), (2, 4))           # K = 256, every code in every block
    scales = np.array([[0.5, 0.25, 2.0, 0.0078125], [1.0, 4.0, 0.125, 0.03125]], np.float16)
    got = O.dequantize_fgq(codes, scales.view(np.uint16), 64).view(np.float16).astype(np.float64)
    vals = np.array([MAGS[c & 31] * (-1 if c & 32 else 1) for c in range(64)])
    for n in range(2):
        for g in range(4):
            assert np.array_equal(got[n, 64 * g:64 * (g + 1)], float(scales[n, g]) * vals)


def test_fgq_linear_bruteforce_fractions_tiny():
    rng = np.random.default_rng(23)
    M, N, K, block = 2, 3, 12, 4
    X = rng.standard_normal((M, K)).astype(np.float16)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    scales = rng.integers(0x1000, 0x3C00, (N, K // block)).astype(np.uint16)
    Y = O.linear_fgq(X, codes, scales, block)
    for m in range(M):
        for n in range(N):
            exact = Fraction(0)
            for k in range(K):
                S = Fraction(float(scales[n, k // block:k // block + 1].view(np.float16)[0]))
                exact += S * Fraction(float(X[m, k])) * Fraction(MAGS[codes[n, k] & 31]) * (-1 if codes[n, k] & 32 else 1)
            assert abs(Y[m, n] - float(exact)) <= 1e-13 * max(1.0, abs(float(exact)))


def test_fgq_linear_equals_numpy_matmul_when_everything_is_exact():
    # small integers and power-of-two scales: every product, block sum and total is exact in
    # double, so the definition must equal numpy's float64 matmul on the scaled weights
    rng = np.random.default_rng(24)
    M, N, K, block = 4, 5, 256, 64
    X = rng.integers(-8, 9, (M, K)).astype(np.float16)
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    scales = (2.0 ** rng.integers(-6, 3, (N, K // block))).astype(np.float16)
    Wv = np.array([[MAGS[c & 31] * (-1 if c & 32 else 1) for c in row] for row in codes])
    Ws = Wv * scales.astype(np.float64).repeat(block, axis=1)
    assert np.array_equal(O.linear_fgq(X, codes, scales.view(np.uint16), block), X.astype(np.float64) @ Ws.T)


def test_fgq_linear_scale_multiplies_the_block_sum_not_the_rounded_weight():
    # S * 7 needs 13 significant bits: the exact product must survive (no fp16 rounding of S*v)
    S = np.array([[0.0999755859375, 0.5]], np.float16)
    codes = np.array([[23, 0, 0, 0, 12, 12, 12, 12]], np.uint8)
    X = np.array([[1, 0, 0, 0, 1, 1, 1, 1]], np.float16)
    Y = O.linear_fgq(X, codes, S.view(np.uint16), 4)
    assert Y[0, 0] == float(S[0, 0]) * 7.0 + 0.5 * 4.0


# ------------------------------------------------------------------ FP5 E3M1 ("4+1")

GOLDEN5 = os.path.join(os.path.dirname(__file__), "golden", "e3m1_magnitudes.txt")
MAGS5 = [float(l.split()[3]) for l in open(GOLDEN5) if l.strip() and not l.startswith("#")]


def test_e3m1_values_closed_form_and_subset_of_e3m2():
    assert len(MAGS5) == 16 and max(MAGS5) == 24.0 == 2.0 ** 4 * 1.5
    for c in range(32):
        s, E, m = c >> 4, (c >> 1) & 7, c & 1
        x = Fraction(2) ** (E - 3) * (1 + Fraction(m, 2)) if E else Fraction(1, 4) * Fraction(m, 2)
        assert Fraction(O.e3m1_value(c)) == (-x if s else x)
        assert abs(O.e3m1_value(c)) == MAGS5[c & 15]
        # same sign and exponent, mantissa bits "m0", in the six-bit format
        assert O.e3m1_value(c) == O.e3m2_value(s << 5 | E << 2 | m << 1) or (c == 16 and O.e3m1_value(c) == 0.0)
    assert np.signbit(O.e3m1_value(16))


def test_e3m1_bias_shift_identity_numpy_fp16():
    # Eq. 5 for the five-bit format: bits s<<15 | eee<<10 | m<<9 read as fp16, times 2^12, are the value
    for c in range(32):
        bits = O.bias_shift_bits5(c)
        assert bits == ((c >> 4) << 15 | ((c >> 1) & 7) << 10 | (c & 1) << 9)
        h = np.array([bits], np.uint16).view(np.float16).astype(np.float64)[0]
        assert h * 4096.0 == O.e3m1_value(c)
        if ((c >> 1) & 7) == 0 and (c & 1):
            assert ((bits >> 10) & 31) == 0 and (bits & 0x3FF)        # an fp16 subnormal


def test_e3m1_quantize_bruteforce_and_invariants():
    rng = np.random.default_rng(51)
    N, K = 6, 96
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0, :] = 0                                   # zero row
    W[1, 5] = np.float16(-1e-7)                   # tiny negative keeps its sign
    codes, scales = O.quantize5(W)
    amax = np.abs(W.astype(np.float64)).max(axis=1)
    assert np.array_equal(scales.view(np.float16), (amax / 24.0).astype(np.float16))
    for n in range(N):
        S = Fraction(float(scales[n:n + 1].view(np.float16)[0]))
        for k in range(K):
            w = Fraction(float(W[n, k]))
            c = int(codes[n, k])
            assert (c >> 4) == int(np.signbit(W[n, k]))
            if S == 0:
                assert (c & 15) == 0
                continue
            d = [abs(abs(w) / S - Fraction(MAGS5[i])) for i in range(16)]
            best = min(d)
            cands = [i for i in range(16) if d[i] == best]
            want = cands[0] if len(cands) == 1 else [i for i in cands if i % 2 == 0][0]
            assert (c & 15) == want
    # the row maximum sits on the largest code
    assert all((codes[n, np.abs(W[n].astype(np.float64)).argmax()] & 15) == 15 for n in range(1, N))
    # idempotent on the grid: rows S0 * value(c) come back as c (including -0)
    S0 = 2.0 ** -5
    grid = np.array([[O.e3m1_value(c) * S0 for c in range(32)]], np.float16)
    grid.view(np.uint16)[0, 16] = 0x8000
    c2, s2 = O.quantize5(grid)
    assert c2[0].tolist() == list(range(32)) and float(s2.view(np.float16)[0]) == S0
    hi4, lo1 = O.split41(c2)
    assert np.array_equal(hi4, c2 >> 1) and np.array_equal(lo1, c2 & 1)


def test_e3m1_ties_go_to_even_code():
    # S = 1/8 exactly (amax = 3): w = S * midpoint of two neighbouring magnitudes
    mids = [(MAGS5[i] + MAGS5[i + 1]) / 2 for i in range(15)]
    row = np.array([[3.0] + [m / 8.0 for m in mids]], np.float16)
    assert all(float(v) * 8.0 == m for v, m in zip(row[0, 1:], mids))      # representable: real ties
    codes, scales = O.quantize5(row)
    assert float(scales.view(np.float16)[0]) == 0.125
    for i, c in enumerate(codes[0, 1:]):
        assert (c & 15) == (i if i % 2 == 0 else i + 1)


def test_e3m1_dequantize_and_linear_vs_numpy():
    rng = np.random.default_rng(52)
    scales = rng.integers(1, 0x7000, 40).astype(np.uint16)
    codes = np.tile(np.arange(32, dtype=np.uint8), (scales.size, 1))
    vals = np.array([O.e3m1_value(c) for c in range(32)])
    ref = (scales.view(np.float16).astype(np.float64)[:, None] * vals[None, :]).astype(np.float16)
    assert np.array_equal(O.dequantize5(codes, scales), ref.view(np.uint16))
    M, N, K = 4, 5, 64
    X = rng.integers(-8, 9, (M, K)).astype(np.float16)
    codes = rng.integers(0, 32, (N, K), dtype=np.uint8)
    sc = np.array([2.0 ** -k for k in range(N)], np.float16)
    Wv = vals[codes]
    assert np.array_equal(O.linear5(X, codes, sc.view(np.uint16)), (X.astype(np.float64) @ Wv.T) * sc.astype(np.float64)[None, :])


# ---- bf16 activations (Section 2: FP16 or BF16 around the FP6 weights)

def _bf16_value(bits: int) -> Fraction:
    """bf16 bit pattern -> exact value, from the format's definition (1-8-7, bias 127)."""
    s, e, m = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
    assert e != 0xFF
    mag = Fraction(m, 128) * Fraction(2) ** (-126) if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
    return -mag if s else mag


def test_bf16_to_double_is_the_format_definition_for_every_finite_pattern():
    for bits in range(0x10000):
        if (bits >> 7) & 0xFF == 0xFF:
            continue
        assert Fraction(O.bf16_to_double(bits)) == _bf16_value(bits), hex(bits)
    assert math.copysign(1.0, O.bf16_to_double(0x8000)) == -1.0


def test_double_to_bf16_rounds_to_nearest_ties_to_even():
    # every finite pattern is a fixed point; the midpoint to the next pattern goes to the even one;
    # just below / above the midpoint goes down / up
    for bits in list(range(0, 0x7F80, 7)) + [0x0001, 0x007F, 0x0080, 0x7F7E]:
        v = _bf16_value(bits)
        assert O.double_to_bf16(float(v)) == bits
        assert O.double_to_bf16(-float(v)) == bits | 0x8000          # -0.0 for the zero pattern
        if bits + 1 < 0x7F80:
            mid = (v + _bf16_value(bits + 1)) / 2
            even = bits if bits % 2 == 0 else bits + 1
            assert O.double_to_bf16(float(mid)) == even, hex(bits)
            eps = (_bf16_value(bits + 1) - v) / 1024
            assert O.double_to_bf16(float(mid - eps)) == bits
            assert O.double_to_bf16(float(mid + eps)) == bits + 1
    # a library routine on values it converts without a second rounding (float32-exact inputs)
    import torch
    x = np.random.default_rng(31).standard_normal(5000).astype(np.float32) * np.float32(37.0)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([O.double_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_linear_bf16_is_linear_on_values_both_types_hold_and_bruteforce():
    rng = np.random.default_rng(32)
    M, N, K = 3, 4, 40
    codes = rng.integers(0, 64, (N, K), dtype=np.uint8)
    scales = rng.integers(0x1000, 0x3C00, N).astype(np.uint16)
    # multiples of 1/8 up to 8: exact in fp16 and in bf16
    Xv = rng.integers(-64, 65, (M, K)) / 8.0
    X16 = Xv.astype(np.float16)
    Xb = np.array([[O.double_to_bf16(float(v)) for v in row] for row in Xv], dtype=np.uint16)
    assert np.array_equal(O.linear_bf16(Xb, codes, scales), O.linear(X16, codes, scales))
    # arbitrary bf16 patterns (values fp16 cannot hold) against exact rational arithmetic
    Xb = rng.integers(0x3000, 0x4800, (M, K)).astype(np.uint16) | (rng.integers(0, 2, (M, K)).astype(np.uint16) << 15)
    Y = O.linear_bf16(Xb, codes, scales)
    for m in range(M):
        for n in range(N):
            S = Fraction(float(scales[n:n + 1].view(np.float16)[0]))
            exact = S * sum(_bf16_value(int(Xb[m, k])) * Fraction(MAGS[codes[n, k] & 31]) * (-1 if codes[n, k] & 32 else 1)
                            for k in range(K))
            assert abs(Y[m, n] - float(exact)) <= 1e-13 * max(1.0, abs(float(exact)))
