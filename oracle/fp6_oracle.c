/*
 * CPU oracle for the W6A16 linear layer of ZeroQuant(4+2) (arXiv 2312.08583).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * obviously-correct statement of what the method computes, written from the
 * paper.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it.  It shares no code, header, table or helper
 * with the HIP library and knows nothing about that library's physical plane
 * layout: it works on one 6-bit code per weight and on the *logical* 4+2 split.
 *
 * Every quantity that the paper defines exactly is evaluated here in exact
 * integer arithmetic (fp16 numbers are integer multiples of 2^-24), so that no
 * question of intermediate rounding can arise.  The linear layer itself is the
 * plain triple loop in double precision.
 *
 *   value set ........ Section 4, Eq. 2 (sign, e=3 exponent bits, bias 2^(e-1)-1 = 3,
 *                      mantissa in [0,2)); max magnitude 28 = 2^4 * 1.75; no NaN/inf
 *                      codes (Section 4 footnote); exponent field 0 = subnormal,
 *                      zero included (Section 5.2 footnote).
 *   quantizer ........ Section 4, Eq. 3: W ~ S * W_fp6 with S = max|W| / 28, one S per
 *                      row of W (coarse-grained = row-wise, Section 3 / Appendix A),
 *                      round-to-nearest (Section 3).
 *   4+2 split ........ Section 5.1: first 4 bits = sign + 3-bit exponent, remaining
 *                      2 bits = mantissa.
 *   bias shift ....... Section 5.2, Eq. 5: the same 6 bits read with exponent bias 15
 *                      are an fp16 bit pattern (pure padding) whose value is the FP6
 *                      value times 2^-12; the 2^12 moves into the scale.
 *   linear ........... Section 5.2: for row-wise scales the scale multiplies the
 *                      finished accumulation; for fine-grained (block-k) scales it
 *                      multiplies each block's product sum before the accumulation.
 *   bf16 activations . Section 2 names BF16 beside FP16 as the type around the FP6
 *                      weights: fp6o_linear_bf16 is the same definition on bf16 X; the two
 *                      conversions (pattern -> value, value -> nearest pattern, ties to
 *                      even) use <math.h> on doubles and are pinned by the tests against the
 *                      format's definition.
 *
 * Readings taken where the paper is silent (listed again in the design notes):
 *   - round-to-nearest ties go to the even magnitude code (IEEE default);
 *   - max|W|/28 and w/S are real-number quotients, rounded once;
 *   - |w/S| > 28 (possible because S was rounded) saturates to 28;
 *   - the sign bit of the code is the sign bit of w (tiny negatives give -0);
 *   - S == 0 (all-zero row or quotient rounding to zero) gives magnitude code 0;
 *   - non-finite weights are rejected (FP6 has no code for them).
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define FP6O_OK 0
#define FP6O_ERR_NONFINITE (-5)
#define FP6O_ERR_ARG (-1)

/* ------------------------------------------------------------------ fp16 */

/* |h| as an integer count of 2^-24 (the fp16 subnormal quantum).  Finite h only. */
static int64_t half_abs_units(uint16_t h)
{
    int e = (h >> 10) & 0x1F;
    int64_t f = h & 0x3FF;
    if (e == 0) return f;                    /* subnormal: f * 2^-24            */
    return (f | 0x400) << (e - 1);           /* (1024+f) * 2^(e-15-10) / 2^-24  */
}

static int half_is_finite(uint16_t h) { return ((h >> 10) & 0x1F) != 0x1F; }

/* exact fp16 -> double */
double fp6o_half_to_double(uint16_t h)
{
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0x1F) {
        v = f ? (0.0 / 0.0) : (1.0 / 0.0);
    } else {
        /* 2^-24 * integer: exact in double */
        v = (double)half_abs_units(h) * (1.0 / 16777216.0);
    }
    return (h & 0x8000) ? -v : v;
}

/*
 * Round the non-negative rational  num / (den * 2^24)  to the nearest fp16,
 * ties to the even significand, overflow to infinity (IEEE 754
 * roundTiesToEven).  Returns the 15 magnitude bits.  den > 0.
 * The fp16 grid, in units of 2^-24, is { q * 2^x : 0 <= q < 2^11, x >= 0 }.
 */
static uint16_t round_units_to_half(int64_t num, int64_t den)
{
    int x = 0;
    /* smallest x with num / (den * 2^x) < 2^11 */
    while (x < 40 && num >= ((den << x) << 11)) x++;
    int64_t d = den << x;
    int64_t q = num / d, rem = num % d;
    if (2 * rem > d || (2 * rem == d && (q & 1))) q++;
    if (q == 2048) { q = 1024; x++; }
    /* value = q * 2^x units of 2^-24 */
    if (q < 1024) {
        /* only possible for x == 0: subnormal (or zero) */
        return (uint16_t)q;
    }
    int e = x + 1;                 /* biased exponent: (1024+f)*2^(e-1) units */
    if (e >= 0x1F) return 0x7C00;  /* overflow -> inf */
    return (uint16_t)((e << 10) | (q & 0x3FF));
}

/* RNE_fp16( num / (den * 2^24) ) for num >= 0, den > 0: the rounding helper on its
 * own, exposed so that tests can pin it against a library's fp16 rounding. */
uint16_t fp6o_round_ratio_to_half(int64_t num, int64_t den)
{
    if (num < 0 || den <= 0) return 0x7E00;
    return round_units_to_half(num, den);
}

/* ------------------------------------------------------------------ E3M2 */

/* 16 * magnitude of the 5-bit magnitude code  eee mm  (Eq. 2 with e=3, b=3):
 *   eee == 0 : subnormal, 2^(1-3) * (mm/4)           = mm / 16
 *   else     : normal,    2^(eee-3) * (1 + mm/4)                          */
static int mag16(int c5)
{
    int e = (c5 >> 2) & 7, m = c5 & 3;
    if (e == 0) return m;
    return (4 + m) << (e - 1);     /* 16 * 2^(e-3) * (4+m)/4 */
}

/* value of the 6-bit code  s eee mm */
double fp6o_e3m2_value(int code)
{
    double v = (double)mag16(code & 31) / 16.0;
    return (code & 32) ? -v : v;
}

/* Eq. 5: the code's bits re-read with bias 15 are these fp16 bits
 * (sign -> bit 15, eee -> low three exponent bits, mm -> top two mantissa bits);
 * fp16(bits) * 2^12 == fp6o_e3m2_value(code). */
uint16_t fp6o_bias_shift_bits(int code)
{
    int s = (code >> 5) & 1, e = (code >> 2) & 7, m = code & 3;
    return (uint16_t)((s << 15) | (e << 10) | (m << 8));
}

/* ------------------------------------------------------------- quantizer */

/* S = RNE_fp16( max|w| / 28 ) for one row (Eq. 3 and the line below it). */
int fp6o_row_scale(const uint16_t *w, int64_t K, uint16_t *S)
{
    int64_t amax = 0;
    for (int64_t k = 0; k < K; k++) {
        if (!half_is_finite(w[k])) return FP6O_ERR_NONFINITE;
        int64_t a = half_abs_units(w[k]);
        if (a > amax) amax = a;
    }
    *S = round_units_to_half(amax, 28);
    return FP6O_OK;
}

/* nearest E3M2 magnitude code to |w| / S; exact; ties -> even code */
static int nearest_mag_code(int64_t w_units, int64_t s_units)
{
    if (s_units == 0) return 0;
    int best = 0;
    int64_t best_d = -1;
    for (int c = 0; c < 32; c++) {
        /* | |w|/S - mag | * 16 * S  in units of 2^-24 */
        int64_t d = 16 * w_units - s_units * (int64_t)mag16(c);
        if (d < 0) d = -d;
        if (best_d < 0 || d < best_d || (d == best_d && (c & 1) == 0 && (best & 1) == 1)) {
            best = c;
            best_d = d;
        }
    }
    return best;   /* |w|/S > 28 lands on c = 31: saturation */
}

/* W fp16 bits [N,K] row-major -> codes [N,K] (one byte each, 0..63), scales fp16 bits [N] */
int fp6o_quantize(const uint16_t *W, int64_t N, int64_t K, uint8_t *codes, uint16_t *scales)
{
    if (!W || !codes || !scales || N < 0 || K < 0) return FP6O_ERR_ARG;
    int status = FP6O_OK;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        const uint16_t *w = W + n * K;
        uint16_t S;
        if (fp6o_row_scale(w, K, &S) != FP6O_OK) {
#pragma omp atomic write
            status = FP6O_ERR_NONFINITE;
            continue;
        }
        scales[n] = S;
        int64_t s_units = half_abs_units(S);
        for (int64_t k = 0; k < K; k++) {
            int c5 = nearest_mag_code(half_abs_units(w[k]), s_units);
            codes[n * K + k] = (uint8_t)(((w[k] >> 15) << 5) | c5);
        }
    }
    return status;
}

/* ------------------------------------------------------------- 4+2 split */

/* Section 5.1: first sub-number = leading 4 bits (sign, exponent), second = last 2 (mantissa) */
void fp6o_split42(const uint8_t *codes, int64_t count, uint8_t *hi4, uint8_t *lo2)
{
    for (int64_t i = 0; i < count; i++) {
        hi4[i] = (uint8_t)((codes[i] >> 2) & 0xF);
        lo2[i] = (uint8_t)(codes[i] & 0x3);
    }
}

void fp6o_join42(const uint8_t *hi4, const uint8_t *lo2, int64_t count, uint8_t *codes)
{
    for (int64_t i = 0; i < count; i++)
        codes[i] = (uint8_t)(((hi4[i] & 0xF) << 2) | (lo2[i] & 0x3));
}

/* ------------------------------------------------------------ dequantize */

/* W_hat[n,k] = RNE_fp16( S_n * value(code) )  (Eq. 3 read right to left) */
void fp6o_dequantize(const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K,
                     uint16_t *W_hat)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        int64_t s_units = half_abs_units(scales[n]);
        for (int64_t k = 0; k < K; k++) {
            int c = codes[n * K + k];
            /* S * mag = s_units * mag16 / 16 units of 2^-24 */
            uint16_t mag = round_units_to_half(s_units * (int64_t)mag16(c & 31), 16);
            W_hat[n * K + k] = (uint16_t)(((c >> 5) << 15) | mag);
        }
    }
}

/* ---------------------------------------------------------------- linear */

/* Y[m,n] = S_n * sum_k X[m,k] * value(code[n,k]), double accumulation, the scale
 * applied to the finished sum (Section 5.2, row-wise case).  Y is [M,N] row-major. */
void fp6o_linear(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales,
                 int64_t N, int64_t K, double *Y)
{
    double *Xd = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    for (int64_t i = 0; i < M * K; i++) Xd[i] = fp6o_half_to_double(X[i]);
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; n++) {
            for (int64_t k = 0; k < K; k++) wrow[k] = fp6o_e3m2_value(codes[n * K + k]);
            double S = fp6o_half_to_double(scales[n]);
            for (int64_t m = 0; m < M; m++) {
                double acc = 0.0;
                const double *x = Xd + m * K;
                for (int64_t k = 0; k < K; k++) acc += x[k] * wrow[k];
                Y[m * N + n] = S * acc;
            }
        }
        free(wrow);
    }
    free(Xd);
}

/* ------------------------------------------------ bf16 activations */

/*
 * bf16 (1 sign, 8 exponent, 7 mantissa bits) is the upper half of an IEEE single: the value of a
 * bit pattern b is that of the single with bits b << 16 (Section 2 names BF16 beside FP16 as the
 * type around the FP6 weights).
 */
double fp6o_bf16_to_double(uint16_t b)
{
    union { uint32_t u; float f; } v;
    v.u = (uint32_t)b << 16;
    return (double)v.f;
}

/*
 * A double rounded to bf16, round to nearest, ties to the even mantissa; finite inputs inside the
 * bf16 range only (the results of a linear layer).  Written out on the value, not on float bits:
 * the spacing of bf16 numbers in the binade of x is 2^(floor(log2|x|) - 7), and subnormals
 * (|x| < 2^-126) have spacing 2^-133.
 */
uint16_t fp6o_double_to_bf16(double x)
{
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    double a = fabs(x);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = f * 2^e, 0.5 <= f < 1  ->  floor(log2 a) = e - 1 */
    int ex = e - 1;
    if (ex < -126) ex = -126;           /* subnormal range shares the spacing of the lowest binade */
    double q = ldexp(a, 7 - ex);        /* in units of the spacing: 128 <= q < 256 for normal numbers */
    double r = nearbyint(q);            /* the default rounding mode is to nearest, ties to even */
    uint32_t m = (uint32_t)r;
    uint32_t bits;
    if (ex == -126 && m < 128u) {
        bits = m;                       /* subnormal: exponent field 0 */
    } else {
        if (m == 256u) { m = 128u; ex += 1; }
        bits = ((uint32_t)(ex + 127) << 7) | (m - 128u);
    }
    return (uint16_t)(sign | (uint16_t)bits);
}

/* fp6o_linear with X given as bf16 bit patterns: the same definition, Y in double. */
void fp6o_linear_bf16(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales,
                      int64_t N, int64_t K, double *Y)
{
    double *Xd = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    for (int64_t i = 0; i < M * K; i++) Xd[i] = fp6o_bf16_to_double(X[i]);
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; n++) {
            for (int64_t k = 0; k < K; k++) wrow[k] = fp6o_e3m2_value(codes[n * K + k]);
            double S = fp6o_half_to_double(scales[n]);
            for (int64_t m = 0; m < M; m++) {
                double acc = 0.0;
                const double *x = Xd + m * K;
                for (int64_t k = 0; k < K; k++) acc += x[k] * wrow[k];
                Y[m * N + n] = S * acc;
            }
        }
        free(wrow);
    }
    free(Xd);
}

/* ------------------------------------------------ fine-grained (block-k) scales */

/*
 * Fine-grained quantization (Section 3, "FGQ"; Appendix A, "block-k quantization: for
 * every k elements, they have their own scaling factor"): a row of W is cut into blocks
 * of `block` consecutive elements along K, and each block is quantized exactly like a
 * whole row above, with its own S = RNE_fp16(max|w| / 28) (Eq. 3).  block == K is the
 * row-wise scheme.  Logical shapes: codes [N,K]; scales [N, K/block] row-major.
 */
int fp6o_quantize_fgq(const uint16_t *W, int64_t N, int64_t K, int64_t block, uint8_t *codes, uint16_t *scales)
{
    if (!W || !codes || !scales || N < 0 || K < 0 || block <= 0 || K % block != 0) return FP6O_ERR_ARG;
    const int64_t G = K / block;
    int status = FP6O_OK;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        for (int64_t g = 0; g < G; g++) {
            const uint16_t *w = W + n * K + g * block;
            uint16_t S;
            if (fp6o_row_scale(w, block, &S) != FP6O_OK) {
#pragma omp atomic write
                status = FP6O_ERR_NONFINITE;
                continue;
            }
            scales[n * G + g] = S;
            int64_t s_units = half_abs_units(S);
            for (int64_t k = 0; k < block; k++) {
                int c5 = nearest_mag_code(half_abs_units(w[k]), s_units);
                codes[n * K + g * block + k] = (uint8_t)(((w[k] >> 15) << 5) | c5);
            }
        }
    }
    return status;
}

/* W_hat[n,k] = RNE_fp16( S[n, k/block] * value(code) ) */
void fp6o_dequantize_fgq(const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, int64_t block,
                         uint16_t *W_hat)
{
    const int64_t G = K / block;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        for (int64_t k = 0; k < K; k++) {
            int64_t s_units = half_abs_units(scales[n * G + k / block]);
            int c = codes[n * K + k];
            uint16_t mag = round_units_to_half(s_units * (int64_t)mag16(c & 31), 16);
            W_hat[n * K + k] = (uint16_t)(((c >> 5) << 15) | mag);
        }
    }
}

/* Y[m,n] = sum_g S[n,g] * ( sum_{k in block g} X[m,k] * value(code[n,k]) ): the scale
 * multiplies each block's product sum before the blocks are accumulated (Section 5.2,
 * fine-grained case).  Double precision throughout. */
void fp6o_linear_fgq(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales,
                     int64_t N, int64_t K, int64_t block, double *Y)
{
    const int64_t G = K / block;
    double *Xd = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    for (int64_t i = 0; i < M * K; i++) Xd[i] = fp6o_half_to_double(X[i]);
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; n++) {
            for (int64_t k = 0; k < K; k++) wrow[k] = fp6o_e3m2_value(codes[n * K + k]);
            for (int64_t m = 0; m < M; m++) {
                const double *x = Xd + m * K;
                double y = 0.0;
                for (int64_t g = 0; g < G; g++) {
                    double acc = 0.0;
                    for (int64_t k = g * block; k < (g + 1) * block; k++) acc += x[k] * wrow[k];
                    y += fp6o_half_to_double(scales[n * G + g]) * acc;
                }
                Y[m * N + n] = y;
            }
        }
        free(wrow);
    }
    free(Xd);
}

/* ------------------------------------------------------------- FP5 E3M1, "4+1" */

/*
 * The five-bit format the paper names beside FP6 (Section 4: "similar setting is defined
 * for FP5 E3M1"; Section 6: the 4+2 technique adapts to 5-bit quantization).  Eq. 2 with
 * e = 3, bias 3 and ONE mantissa bit: code  s eee m  (0..31);
 *   eee == 0 : subnormal, 2^(1-3) * (m/2) = m / 8          (0 and 0.125)
 *   else     : normal,    2^(eee-3) * (1 + m/2)
 * Largest magnitude 2^4 * 1.5 = 24, so the scale is S = RNE_fp16(max|w| / 24) (Eq. 3 with
 * the format's own maximum).  Rounding, ties, saturation, signs and zero scales follow the
 * same readings as the six-bit quantizer above.  The split is 4 + 1: sign and exponent, and
 * the mantissa bit.  Bias shift (Eq. 5): bits s<<15 | eee<<10 | m<<9 are value * 2^-12.
 */
static int mag8_e3m1(int c4)     /* 8 * magnitude of the 4-bit magnitude code  eee m */
{
    int e = (c4 >> 1) & 7, m = c4 & 1;
    if (e == 0) return m;
    return (2 + m) << (e - 1);   /* 8 * 2^(e-3) * (2+m)/2 */
}

double fp5o_e3m1_value(int code)
{
    double v = (double)mag8_e3m1(code & 15) / 8.0;
    return (code & 16) ? -v : v;
}

uint16_t fp5o_bias_shift_bits(int code)
{
    int s = (code >> 4) & 1, e = (code >> 1) & 7, m = code & 1;
    return (uint16_t)((s << 15) | (e << 10) | (m << 9));
}

static int nearest_mag_code_e3m1(int64_t w_units, int64_t s_units)
{
    if (s_units == 0) return 0;
    int best = 0;
    int64_t best_d = -1;
    for (int c = 0; c < 16; c++) {
        /* | |w|/S - mag | * 8 * S  in units of 2^-24 */
        int64_t d = 8 * w_units - s_units * (int64_t)mag8_e3m1(c);
        if (d < 0) d = -d;
        if (best_d < 0 || d < best_d || (d == best_d && (c & 1) == 0 && (best & 1) == 1)) {
            best = c;
            best_d = d;
        }
    }
    return best;   /* |w|/S > 24 lands on c = 15: saturation */
}

/* W fp16 bits [N,K] -> codes [N,K] (0..31), scales fp16 bits [N] (row-wise) */
int fp5o_quantize(const uint16_t *W, int64_t N, int64_t K, uint8_t *codes, uint16_t *scales)
{
    if (!W || !codes || !scales || N < 0 || K < 0) return FP6O_ERR_ARG;
    int status = FP6O_OK;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        const uint16_t *w = W + n * K;
        int64_t amax = 0;
        int bad = 0;
        for (int64_t k = 0; k < K; k++) {
            if (!half_is_finite(w[k])) bad = 1;
            int64_t a = half_abs_units(w[k]);
            if (a > amax) amax = a;
        }
        if (bad) {
#pragma omp atomic write
            status = FP6O_ERR_NONFINITE;
            continue;
        }
        uint16_t S = round_units_to_half(amax, 24);
        scales[n] = S;
        int64_t s_units = half_abs_units(S);
        for (int64_t k = 0; k < K; k++) {
            int c4 = nearest_mag_code_e3m1(half_abs_units(w[k]), s_units);
            codes[n * K + k] = (uint8_t)(((w[k] >> 15) << 4) | c4);
        }
    }
    return status;
}

/* 4 + 1 split: first sub-number = sign and exponent, second = the mantissa bit */
void fp5o_split41(const uint8_t *codes, int64_t count, uint8_t *hi4, uint8_t *lo1)
{
    for (int64_t i = 0; i < count; i++) {
        hi4[i] = (uint8_t)((codes[i] >> 1) & 0xF);
        lo1[i] = (uint8_t)(codes[i] & 0x1);
    }
}

/* W_hat[n,k] = RNE_fp16( S_n * value(code) ) */
void fp5o_dequantize(const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, uint16_t *W_hat)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; n++) {
        int64_t s_units = half_abs_units(scales[n]);
        for (int64_t k = 0; k < K; k++) {
            int c = codes[n * K + k];
            uint16_t mag = round_units_to_half(s_units * (int64_t)mag8_e3m1(c & 15), 8);
            W_hat[n * K + k] = (uint16_t)(((c >> 4) << 15) | mag);
        }
    }
}

/* Y[m,n] = S_n * sum_k X[m,k] * value(code[n,k]), double accumulation, scale after the sum */
void fp5o_linear(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales,
                 int64_t N, int64_t K, double *Y)
{
    double *Xd = (double *)malloc(sizeof(double) * (size_t)(M * K > 0 ? M * K : 1));
    for (int64_t i = 0; i < M * K; i++) Xd[i] = fp6o_half_to_double(X[i]);
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; n++) {
            for (int64_t k = 0; k < K; k++) wrow[k] = fp5o_e3m1_value(codes[n * K + k]);
            double S = fp6o_half_to_double(scales[n]);
            for (int64_t m = 0; m < M; m++) {
                double acc = 0.0;
                const double *x = Xd + m * K;
                for (int64_t k = 0; k < K; k++) acc += x[k] * wrow[k];
                Y[m * N + n] = S * acc;
            }
        }
        free(wrow);
    }
    free(Xd);
}

/* number of host threads the loops above use */
int fp6o_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
