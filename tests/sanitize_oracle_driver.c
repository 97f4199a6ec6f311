/*
 * Driver for the sanitizer build of the CPU oracle (test infrastructure).
 *
 * Linked against oracle/fp6_oracle.c with -fsanitize=address,undefined, it calls every
 * oracle routine on small seeded inputs - ragged sizes, an all-zero row, the largest and
 * the smallest fp16 magnitudes - and prints one FNV-1a hash per result.  A sanitizer
 * report ends the program with a non-zero status; tests/test_sanitizers.py also checks
 * the hashes against the ordinary build of the oracle fed the same inputs.
 *
 * Inputs: a 64-bit linear congruential generator (x <- x * 6364136223846793005 + 1442695040888963407,
 * output = top 16 bits), the same in the Python test; patterns with an all-ones fp16
 * exponent field have exponent bit 14 cleared, so every input is finite.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double fp6o_half_to_double(uint16_t h);
uint16_t fp6o_round_ratio_to_half(int64_t num, int64_t den);
double fp6o_e3m2_value(int code);
uint16_t fp6o_bias_shift_bits(int code);
int fp6o_quantize(const uint16_t *W, int64_t N, int64_t K, uint8_t *codes, uint16_t *scales);
void fp6o_split42(const uint8_t *codes, int64_t count, uint8_t *hi4, uint8_t *lo2);
void fp6o_join42(const uint8_t *hi4, const uint8_t *lo2, int64_t count, uint8_t *codes);
void fp6o_dequantize(const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, uint16_t *W_hat);
void fp6o_linear(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, double *Y);
double fp6o_bf16_to_double(uint16_t b);
uint16_t fp6o_double_to_bf16(double x);
void fp6o_linear_bf16(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, double *Y);
int fp6o_quantize_fgq(const uint16_t *W, int64_t N, int64_t K, int64_t block, uint8_t *codes, uint16_t *scales);
void fp6o_dequantize_fgq(const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, int64_t block, uint16_t *W_hat);
void fp6o_linear_fgq(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, int64_t block, double *Y);
double fp5o_e3m1_value(int code);
uint16_t fp5o_bias_shift_bits(int code);
int fp5o_quantize(const uint16_t *W, int64_t N, int64_t K, uint8_t *codes, uint16_t *scales);
void fp5o_split41(const uint8_t *codes, int64_t count, uint8_t *hi4, uint8_t *lo1);
void fp5o_dequantize(const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, uint16_t *W_hat);
void fp5o_linear(const uint16_t *X, int64_t M, const uint8_t *codes, const uint16_t *scales, int64_t N, int64_t K, double *Y);

static uint64_t lcg_state;
static uint16_t next16(void)
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint16_t)(lcg_state >> 48);
}
static uint16_t finite16(void)
{
    uint16_t p = next16();
    if (((p >> 10) & 31) == 31) p &= (uint16_t)~0x4000u;
    return p;
}

static void show(const char *name, const void *data, size_t bytes)
{
    uint64_t h = 1469598103934665603ull;
    const unsigned char *p = (const unsigned char *)data;
    for (size_t i = 0; i < bytes; i++) h = (h ^ p[i]) * 1099511628211ull;
    printf("%s %016llx\n", name, (unsigned long long)h);
}

int main(void)
{
    enum { N = 7, K = 192, M = 3, BLOCK = 64 };
    uint16_t *W = malloc(sizeof(uint16_t) * N * K), *X = malloc(sizeof(uint16_t) * M * K);
    uint8_t *codes = malloc(N * K), *hi = malloc(N * K), *lo = malloc(N * K), *back = malloc(N * K);
    uint16_t *scales = malloc(sizeof(uint16_t) * N * (K / BLOCK)), *What = malloc(sizeof(uint16_t) * N * K);
    double *Y = malloc(sizeof(double) * M * N);
    lcg_state = 231208583u;
    for (int i = 0; i < N * K; i++) W[i] = finite16();
    for (int i = 0; i < M * K; i++) X[i] = (uint16_t)((finite16() & 0xBFFF) | 0x0000);   /* |x| < 2 */
    for (int k = 0; k < K; k++) W[2 * K + k] = (uint16_t)(k & 1 ? 0x8000 : 0);           /* a row of +-0 */
    W[3 * K] = 0x7BFF; W[3 * K + 1] = 0xFBFF; W[3 * K + 2] = 0x0001; W[3 * K + 3] = 0x8001;  /* largest, smallest */
    for (int k = 0; k < K; k++) W[4 * K + k] = (uint16_t)(k % 3);                        /* subnormal row: S rounds to 0 */

    double acc = 0.0;
    for (int c = 0; c < 64; c++) acc += fp6o_e3m2_value(c) * (c + 1) + fp6o_half_to_double(fp6o_bias_shift_bits(c));
    for (int c = 0; c < 32; c++) acc += fp5o_e3m1_value(c) * (c + 1) + fp6o_half_to_double(fp5o_bias_shift_bits(c));
    show("tables", &acc, sizeof acc);
    uint16_t r[4] = {fp6o_round_ratio_to_half(65504ll << 9, 28), fp6o_round_ratio_to_half(1, 28),
                     fp6o_round_ratio_to_half(0, 28), fp6o_round_ratio_to_half((int64_t)1 << 40, 1)};
    show("ratio", r, sizeof r);
    uint16_t b[3] = {fp6o_double_to_bf16(1.00390625), fp6o_double_to_bf16(-3.0e38), fp6o_double_to_bf16(1e-40)};
    double bd = fp6o_bf16_to_double(0x3F80) + fp6o_bf16_to_double(0x8001);
    show("bf16", b, sizeof b);
    show("bf16d", &bd, sizeof bd);

    if (fp6o_quantize(W, N, K, codes, scales) != 0) return 3;
    show("q6.codes", codes, N * K);
    show("q6.scales", scales, sizeof(uint16_t) * N);
    fp6o_split42(codes, N * K, hi, lo);
    fp6o_join42(hi, lo, N * K, back);
    if (memcmp(codes, back, N * K)) return 4;
    show("q6.hi", hi, N * K);
    fp6o_dequantize(codes, scales, N, K, What);
    show("q6.what", What, sizeof(uint16_t) * N * K);
    fp6o_linear(X, M, codes, scales, N, K, Y);
    show("q6.y", Y, sizeof(double) * M * N);
    fp6o_linear_bf16(X, M, codes, scales, N, K, Y);
    show("q6.ybf16", Y, sizeof(double) * M * N);
    fp6o_linear(X, 0, codes, scales, N, K, Y);          /* empty batch: nothing read or written */
    fp6o_linear(X, M, codes, scales, 0, K, Y);

    if (fp6o_quantize_fgq(W, N, K, BLOCK, codes, scales) != 0) return 5;
    show("fgq.codes", codes, N * K);
    show("fgq.scales", scales, sizeof(uint16_t) * N * (K / BLOCK));
    fp6o_dequantize_fgq(codes, scales, N, K, BLOCK, What);
    show("fgq.what", What, sizeof(uint16_t) * N * K);
    fp6o_linear_fgq(X, M, codes, scales, N, K, BLOCK, Y);
    show("fgq.y", Y, sizeof(double) * M * N);

    if (fp5o_quantize(W, N, K, codes, scales) != 0) return 6;
    show("q5.codes", codes, N * K);
    show("q5.scales", scales, sizeof(uint16_t) * N);
    fp5o_split41(codes, N * K, hi, lo);
    show("q5.lo", lo, N * K);
    fp5o_dequantize(codes, scales, N, K, What);
    show("q5.what", What, sizeof(uint16_t) * N * K);
    fp5o_linear(X, M, codes, scales, N, K, Y);
    show("q5.y", Y, sizeof(double) * M * N);

    W[5] = 0x7C00;                                       /* +inf: must be rejected, not read past */
    if (fp6o_quantize(W, N, K, codes, scales) == 0) return 7;
    free(W); free(X); free(codes); free(hi); free(lo); free(back); free(scales); free(What); free(Y);
    puts("done");
    return 0;
}
