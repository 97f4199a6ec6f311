/*
 * fp6_linear.h - C ABI of the MI355X (gfx950) W6A16 linear layer of ZeroQuant(4+2),
 * arXiv 2312.08583.
 *
 * The layer: weights are FP6 E3M2 numbers (Section 4, Eq. 2: 1 sign, 3 exponent bits
 * with bias 3, 2 mantissa bits; largest magnitude 28; no NaN/inf; exponent field 0 is
 * subnormal) with one fp16 scale per output channel, S = max|w| / 28 (Section 4, Eq. 3;
 * row-wise = coarse-grained scaling, Section 3).  Each 6-bit code is stored as two
 * sub-numbers in two separate arrays ("4+2", Section 5.1): a 4-bit one (sign + exponent)
 * and a 2-bit one (mantissa).  At run time the two are loaded together, padded into an
 * fp16 bit pattern without exponent arithmetic ("bias shift", Section 5.2, Eq. 5: the
 * bits are read with exponent bias 15 and the factor 2^12 moves into the scale), and
 * contracted with fp16 activations; the scale multiplies the finished accumulation
 * (Section 5.2, row-wise case).
 *
 * Conventions
 *   - W is [N, K] = [out_features, in_features], row-major, as in the paper's kernel
 *     table (Appendix B: weight 5504*2048 times input 2048*8).  X is [M, K] row-major,
 *     Y is [M, N] row-major.  There is no bias term.
 *   - fp16 data are passed as uint16_t bit patterns.
 *   - Every buffer pointer is a DEVICE pointer owned by the caller, 16-byte aligned.
 *     The library never allocates, frees or synchronises; it keeps no global state, with one
 *     exception: the built-in scratch of fp6_linear_static (see there).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream.
 *   - N and K must be positive multiples of FP6_TILE (64).  M >= 1.
 *   - Return value: FP6_OK or a negative fp6_status.  Argument errors are found on the
 *     host before anything is launched, so nothing is written in that case.
 *
 * Physical layout of the planes (layout version 1; opaque to callers, stated here so
 * that it can be checked).  The weight is cut into tiles of 64 rows (n) by 64 columns
 * (k); tile (nb, kb) has index ti = nb * (K/64) + kb and owns 2048 contiguous bytes of
 * the 4-bit plane and 1024 contiguous bytes of the 2-bit plane.  Inside a tile a weight
 * at (nn, kk) = (n % 64, k % 64) belongs to
 *     lane      l = 16 * ((kk % 32) / 8) + (nn % 16)          (0..63, one wavefront)
 *     fragment  f = 2 * (nn / 16) + (kk / 32)                 (0..7)
 *     element   e = kk % 8  =  4 * grp + j   (grp = e / 4, j = e % 4), kept in byte
 *               b = 2 * (j % 2) + j / 2 of its dword
 *   so that one lane's eight elements of a fragment are the eight consecutive-k fp16
 *   operands that lane feeds to v_mfma_f32_16x16x32_f16 for a 16(n) x 32(k) block.
 *   4-bit plane: byte ti*2048 + (f/4)*1024 + l*16 + (f%4)*4 + b holds, for the two
 *     elements b (grp 0) and 4+b (grp 1):  bit0 = sign(grp0), bit1 = sign(grp1),
 *     bits 4..2 = exponent(grp0), bits 7..5 = exponent(grp1).
 *   2-bit plane: byte ti*1024 + l*16 + (f/2)*4 + b holds the mantissas of elements b and
 *     4+b of fragments f (even) and f+1: bits 1..0 = (f, grp0), 3..2 = (f, grp1),
 *     5..4 = (f+1, grp0), 7..6 = (f+1, grp1).
 *   A wavefront therefore fetches a whole tile with three coalesced 128-bit loads per
 *   lane, and turns four weights at a time into the byte s00eeemm (the top byte of the
 *   bias-15 fp16 pattern) with a handful of 32-bit logic operations.
 */
#ifndef FP6_LINEAR_H
#define FP6_LINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FP6_TILE 64            /* N and K granularity */
#define FP6_LAYOUT_VERSION 1

typedef enum {
    FP6_OK = 0,
    FP6_ERR_NULL = -1,       /* a required pointer is NULL                                  */
    FP6_ERR_SHAPE = -2,      /* M, N or K not positive, or N, K not multiples of FP6_TILE    */
    FP6_ERR_ALIGN = -3,      /* a buffer pointer is not 16-byte aligned                      */
    FP6_ERR_WORKSPACE = -4,  /* workspace missing or smaller than fp6_linear_workspace_bytes */
    FP6_ERR_VARIANT = -5,    /* kernel variant / split request not valid for this shape      */
    FP6_ERR_HIP = -6,        /* the HIP runtime reported a launch error                      */
    FP6_ERR_SCRATCH = -7     /* fp6_linear_static: the shape needs more than its built-in scratch */
} fp6_status;

/* kernel families behind fp6_linear (see fp6_linear_variant) */
typedef enum {
    FP6_VARIANT_AUTO = 0,
    FP6_VARIANT_DECODE = 1,  /* M <= 16: one MFMA row block, K split over the wavefronts of a
                                workgroup (and optionally over workgroups), reduced on chip;
                                on request also M <= 64 (two or four row blocks per wavefront,
                                row-wise FP6 without tuning hints)                            */
    FP6_VARIANT_GEMM = 2     /* any M: activations staged in LDS, wavefronts side by side in N */
} fp6_variant;

/* Layout version of the packed planes written by fp6_quantize_pack. */
int fp6_layout_version(void);

/* Human-readable text for a status code (static storage; never NULL). */
const char *fp6_status_string(int status);

/*
 * Sizes in bytes of the three packed buffers for an [N,K] weight: N*K/2, N*K/4 (together
 * 0.75 byte per weight, Section 5.1) and 2*N.  Host-only; any of the outputs may be NULL.
 */
int fp6_packed_sizes(int64_t N, int64_t K, size_t *hi_bytes, size_t *lo_bytes, size_t *scale_bytes);

/*
 * Offline step (Section 4, Eq. 3; Section 5.1; "performed statically", Section 5.2):
 * per row n, S_n = RNE_fp16(max_k |W[n,k]| / 28); every weight is rounded to the nearest
 * E3M2 value of W/S_n (ties to the even code, saturating at 28, sign bit kept, S_n == 0
 * gives zero codes) and its 6 bits are split into the two planes in the layout above.
 *   W       in   device, fp16 bits [N,K] row-major; must be finite (non-finite entries are
 *                not detected and give unspecified codes, never a fault)
 *   hi_plane out device, N*K/2 bytes (4-bit sub-numbers)
 *   lo_plane out device, N*K/4 bytes (2-bit sub-numbers)
 *   scales  out  device, fp16 bits [N]: the TRUE scale S_n (the 2^12 of the bias shift is
 *                applied inside fp6_linear in fp32, so S need not be below 1)
 */
int fp6_quantize_pack(const uint16_t *W, int64_t N, int64_t K, void *hi_plane, void *lo_plane,
                      uint16_t *scales, void *stream);

/*
 * Test utility: planes -> one code per weight, codes[n*K+k] = s<<5 | eee<<2 | mm (0..63),
 * i.e. the logical 4-bit sub-number is codes>>2 and the 2-bit one is codes&3 (Section 5.1).
 *   codes out device, N*K bytes
 */
int fp6_unpack_codes(const void *hi_plane, const void *lo_plane, int64_t N, int64_t K,
                     uint8_t *codes, void *stream);

/*
 * Test utility: W_hat[n,k] = RNE_fp16(S_n * value(code[n,k]))  (Eq. 3 read backwards),
 * fp16 bits [N,K] row-major, device.
 */
int fp6_dequantize(const void *hi_plane, const void *lo_plane, const uint16_t *scales,
                   int64_t N, int64_t K, uint16_t *W_hat, void *stream);

/*
 * Bytes of device workspace fp6_linear may need for this shape (0 is possible).  When K
 * is cut into slices handled by different workgroups, the workspace is where the slices'
 * fp32 partial sums meet: small ones pairwise in 64-bit slots, large ones through a
 * buffer guarded by one arrival counter per output tile.  CONTRACT: the first
 * FP6_WORKSPACE_ZERO_BYTES bytes (counters and slots) must be zero before the first call
 * that uses the workspace; every call leaves them zero again, so one buffer can be reused
 * by successive calls on the same stream, whatever their shapes.  Calls that share a
 * workspace must not overlap in time.
 */
#define FP6_WORKSPACE_ZERO_BYTES 4259840
size_t fp6_linear_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Hot path (Sections 5.1-5.2): Y[m,n] = fp16( (sum_k X[m,k] * h(code[n,k])) * (S_n * 2^12) )
 * where h is the code's six bits padded into an fp16 (exponent bias 15, Eq. 5), the sum
 * is accumulated in fp32 on the matrix cores, and the row scale is applied once after
 * the accumulation.
 *   X         in  device, fp16 bits [M,K] row-major
 *   hi_plane, lo_plane, scales  in  device, as written by fp6_quantize_pack
 *   Y         out device, fp16 bits [M,N] row-major
 *   workspace     device, >= fp6_linear_workspace_bytes(M,N,K) bytes (may be NULL if that is 0)
 * Nothing is clamped and nothing is checked for finiteness: a result beyond the fp16 range is
 * stored as an infinity, an infinite or NaN activation propagates through its row of Y by the
 * rules of IEEE arithmetic (inf * 0 and inf - inf give NaN), other rows are not affected.
 */
int fp6_linear(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
               const uint16_t *scales, int64_t N, int64_t K, uint16_t *Y,
               void *workspace, size_t workspace_bytes, void *stream);

/*
 * fp6_linear for callers that cannot hand over, or allocate, a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels and
 * same results as fp6_linear(X, M, ..., Y, workspace, ...); the K-slices meet in
 * FP6_STATIC_SCRATCH_BYTES (64 MiB) of device memory that belongs to the library: a static device
 * array, one copy per GPU the library is used on, held until the process ends.  The call allocates
 * and frees nothing and never synchronises.
 *   - A shape whose plan needs more scratch than that returns FP6_ERR_SCRATCH before anything is
 *     launched (the need is what fp6_linear_workspace_bytes reports; e.g. M = 512 with K split four
 *     ways over 8192 output channels does not fit): use fp6_linear with a workspace there.
 *   - All calls on one GPU share that GPU's scratch, which keeps what the last call left: the
 *     counters and slots at its start are cleared by the first call on a device (a small fill kernel
 *     on `stream`, ahead of the first launch) and left zero by every call, the partial sums are
 *     overwritten before they are read.  Calls that overlap in time on one GPU (different streams,
 *     parallel graph branches) race on it and give wrong results: keep them on one stream.
 *   - A caller that captures graphs makes its first call on each device outside any capture, so that
 *     the one-time fill is executed rather than recorded.
 */
#define FP6_STATIC_SCRATCH_BYTES 67108864
int fp6_linear_static(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
                      const uint16_t *scales, int64_t N, int64_t K, uint16_t *Y, void *stream);

/*
 * Several independent layers on activations of the same height M in one call: the q, k, v projections
 * of an attention block, the gate and up projections of a feed-forward block (Section 5.3 measures the
 * kernel on exactly such feed-forward layers).  Each layer i computes what fp6_linear computes for
 * (X_i, planes_i, scales_i) -> Y_i; the caller states by grouping them that no Y_i is read by another
 * layer of the group and that the Y_i do not overlap.  For M <= 16 and layers that share K the group
 * is ONE kernel launch: the workgroups of all layers start together, so a small layer (a 1024 x 8192
 * k projection: 6 MB, mostly launch and tail when launched alone) rides in the shadow of a large one,
 * and the channel blocks of all layers are planned as one list.  Otherwise the layers are launched one
 * after another on `stream`, exactly as separate fp6_linear calls would be.  Results equal those of
 * separate calls up to fp32 summation order (the K-split of a group may differ from a lone layer's).
 *   problems   host array of `count` (1 .. FP6_GROUP_MAX) descriptions, read during the call only;
 *              every pointer inside is a device pointer with the meaning it has in fp6_linear
 *   workspace  device, >= fp6_linear_group_workspace_bytes(M, problems, count) bytes; same contract
 *              as for fp6_linear (first FP6_WORKSPACE_ZERO_BYTES zero before first use, left zero)
 * Errors as fp6_linear, found on the host before anything is launched; FP6_ERR_SHAPE also for a count
 * outside 1 .. FP6_GROUP_MAX.
 */
#define FP6_GROUP_MAX 4
typedef struct fp6_linear_problem {
    const uint16_t *X;        /* fp16 bits [M,K]                      */
    const void *hi_plane;     /* N*K/2 bytes                          */
    const void *lo_plane;     /* N*K/4 bytes                          */
    const uint16_t *scales;   /* fp16 bits [N]                        */
    int64_t N, K;
    uint16_t *Y;              /* fp16 bits [M,N]                      */
} fp6_linear_problem;
size_t fp6_linear_group_workspace_bytes(int64_t M, const fp6_linear_problem *problems, int count);
int fp6_linear_group(int64_t M, const fp6_linear_problem *problems, int count, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * Same computation with the kernel family and the number of K-slices handled by separate
 * workgroups chosen by the caller (tuning sweeps; tests that compare split and unsplit
 * results).  variant = FP6_VARIANT_AUTO and split_k = 0 reproduce fp6_linear.
 * split_k must divide K/64.  The workspace needed is fp6_linear_variant_workspace_bytes.
 * Bits 8 and up of `variant` carry optional tuning hints (0 = automatic):
 *   FP6_HINT_WAVES(w)   wavefronts per workgroup, decode family: 4 or 8 (the gemm family always uses 8,
 *                       two per SIMD, 64 output channels each)
 *   FP6_HINT_DEPTH(d)   tiles in the per-wavefront prefetch ring, decode family: 2..4
 *   FP6_HINT_BLOCK_M(b) rows of X per workgroup, gemm family: 32, 64 or 128
 *   FP6_HINT_MEET(x)    decode family with split_k > 1: 1 = K-slices meet at an arrival counter,
 *                       2 = pairwise in slots (needs split_k * (N/64) * 256 * M <= 2^22)
 *   FP6_HINT_DEQUANT(x) ablations of the bias shift (Section 5.2): the sub-numbers are turned into the
 *                       fp16 numbers that equal the FP6 values themselves and the row scale is applied
 *                       without the 2^12.  1 = integer arithmetic on the exponent field (+12, FP6
 *                       subnormals special-cased: the traditional dequantization the paper compares
 *                       against); 2 = one fp16 multiply by 2^12 per pair of weights.  Same results as
 *                       the bias shift; they exist to measure what it saves.  Not combinable with
 *                       FP6_HINT_WAVES / FP6_HINT_DEPTH.
 *   FP6_HINT_HALF(x)    decode family: 1 = workgroups own 32 output channels (half a tile) instead of 64,
 *                       2 = never; row-wise FP6 with the bias-shift unpack and four wavefronts only; with it
 *                       FP6_HINT_DEPTH may be 4, 6 or 8
 *   FP6_HINT_WIDTH(b)   gemm family: 64-channel blocks (= wavefronts) per workgroup, 8 or 4 (row-wise FP6,
 *                       bias-shift unpack)
 *   FP6_HINT_KWAYS(2)   gemm family, 128 x 256 blocks (FP6_HINT_BLOCK_M(128) | FP6_HINT_WIDTH(4)): eight wavefronts,
 *                       two sets of four that take alternate k tiles and add their sums in LDS
 * An unsupported combination returns FP6_ERR_VARIANT.
 */
#define FP6_HINT_WAVES(w) ((int)(w) << 8)
#define FP6_HINT_DEPTH(d) ((int)(d) << 12)
#define FP6_HINT_BLOCK_M(b) (((int)(b) / 16) << 16)
#define FP6_HINT_MEET(x) ((int)(x) << 20)
#define FP6_HINT_DEQUANT(x) ((int)(x) << 22)
#define FP6_HINT_HALF(x) ((int)(x) << 24)
#define FP6_HINT_WIDTH(b) ((int)(b) << 26)
#define FP6_HINT_KWAYS(x) (((int)(x) == 2) << 30)
size_t fp6_linear_variant_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int split_k);
int fp6_linear_variant(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
                       const uint16_t *scales, int64_t N, int64_t K, uint16_t *Y,
                       void *workspace, size_t workspace_bytes, void *stream,
                       int variant, int split_k);

/*
 * What a call of the hot path would launch (no passage of the paper: the kernel family, tile and
 * K-split are this library's choices for gfx950).  Host-only, touches no GPU: it runs the same
 * planner as fp6_linear / fp6_linear_variant / fp6_linear_fgq / fp5_linear / fp6_linear_v2(_bf16)
 * and reports the result, so that a change of the planner shows up in tests and benchmark rows.
 *   format   FP6_FORMAT_E3M2 (fp6_linear*), FP6_FORMAT_E3M1 (fp5_linear), FP6_FORMAT_E3M2_V2
 *            (fp6_linear_v2), FP6_FORMAT_E3M2_V2_BF16 (fp6_linear_v2_bf16)
 *   block    0 = one scale per row; else the fine-grained block (FP6_FORMAT_E3M2 only)
 *   variant, split_k   as in fp6_linear_variant (0, 0 = what fp6_linear does)
 * Errors: FP6_ERR_NULL (info), FP6_ERR_SHAPE, FP6_ERR_VARIANT (as the call itself would return).
 */
#define FP6_FORMAT_E3M2 6
#define FP6_FORMAT_E3M1 5
#define FP6_FORMAT_E3M2_V2 7
#define FP6_FORMAT_E3M2_V2_BF16 8
typedef struct fp6_plan_info {
    int variant;            /* FP6_VARIANT_DECODE or FP6_VARIANT_GEMM                                   */
    int split_k;            /* K-slices handled by separate workgroups (1 = K is not split)            */
    int block_m;            /* rows of X per workgroup: gemm 32/64/128; decode 16, 32 or 64             */
    int width;              /* 64-channel blocks per workgroup: gemm 8 or 4; decode 1                   */
    int waves;              /* wavefronts per workgroup                                                */
    int depth;              /* tiles (decode) or stages (gemm) in the prefetch ring                    */
    int half_tiles;         /* decode: 1 = workgroups own 32 channels                                   */
    int meeting;            /* how K-slices are added: 0 none, 1 arrival counter, 2 pairwise slots      */
    int64_t workgroups;     /* launch grid                                                             */
    size_t workspace_bytes; /* what the matching *_workspace_bytes call returns                        */
} fp6_plan_info;
int fp6_linear_plan(int format, int64_t M, int64_t N, int64_t K, int64_t block, int variant, int split_k,
                    fp6_plan_info *info);

/*
 * Fine-grained quantization (Section 3, "FGQ"; Appendix A, block-k quantization): every
 * `block` consecutive elements of a row of W share one scale, S = RNE_fp16(max|w| / 28)
 * over the block (Eq. 3), instead of one scale per row.  In the linear layer the scale
 * multiplies the product sum of its block before the blocks are accumulated (Section 5.2,
 * fine-grained case):
 *     Y[m,n] = fp16( 2^12 * sum_g float(S[n,g]) * ( sum_{k in block g} X[m,k] * h(code[n,k]) ) )
 * with fp32 accumulation inside and across blocks.
 *   block   64, 128, 256, ... (64 times a power of two), dividing K
 *   scales  device, fp16 bits, K/block * N of them; the scale of row n, block g is
 *           scales[g * N + n] (block-major: neighbouring channels are neighbours in memory)
 * Planes, codes and every other convention are those of the row-wise calls above;
 * fp6_unpack_codes serves both.  `variant` and `split_k` as in fp6_linear_variant (0, 0 =
 * automatic); the hints FP6_HINT_WAVES, FP6_HINT_DEPTH, FP6_HINT_DEQUANT and a block_m
 * above 64 are not available with fine-grained scales.
 */
int fp6_quantize_pack_fgq(const uint16_t *W, int64_t N, int64_t K, int64_t block, void *hi_plane,
                          void *lo_plane, uint16_t *scales, void *stream);
int fp6_dequantize_fgq(const void *hi_plane, const void *lo_plane, const uint16_t *scales,
                       int64_t N, int64_t K, int64_t block, uint16_t *W_hat, void *stream);
size_t fp6_linear_fgq_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t block, int variant,
                                      int split_k);
int fp6_linear_fgq(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
                   const uint16_t *scales, int64_t N, int64_t K, int64_t block, uint16_t *Y,
                   void *workspace, size_t workspace_bytes, void *stream, int variant, int split_k);

/*
 * FP5 E3M1, "4+1" (Section 4: a similar setting is defined for FP5 E3M1; Section 6: the
 * technique adapts to 5-bit quantization).  One sign bit, the same three exponent bits
 * with bias 3, ONE mantissa bit; largest magnitude 24, so S_n = RNE_fp16(max|w| / 24); all
 * other quantizer rules as for FP6.  A code is s<<4 | eee<<1 | m (0..31).  The 4-bit plane
 * is exactly the FP6 one (N*K/2 bytes, same layout).  The second plane holds one mantissa
 * bit per weight, N*K/8 bytes - 0.625 byte per weight in total: tile ti owns 512 contiguous
 * bytes, lane l (as above) 8 of them; byte ti*512 + l*8 + (f/4)*4 + b holds, for the
 * fragments f with the same f/4, the mantissa bits of elements b (grp 0) and 4+b (grp 1):
 * bit 2*(f%4) = (f, grp0), bit 2*(f%4) + 1 = (f, grp1).  The bias shift (Eq. 5) pads the
 * bit into position 9 of the fp16 pattern: value * 2^-12 again.
 * Calls mirror the FP6 ones (row-wise scales); `variant` and `split_k` as in
 * fp6_linear_variant, without the hints for waves, depth and dequantization.
 */
int fp5_packed_sizes(int64_t N, int64_t K, size_t *hi_bytes, size_t *lo_bytes, size_t *scale_bytes);
int fp5_quantize_pack(const uint16_t *W, int64_t N, int64_t K, void *hi_plane, void *lo_plane,
                      uint16_t *scales, void *stream);
int fp5_unpack_codes(const void *hi_plane, const void *lo_plane, int64_t N, int64_t K,
                     uint8_t *codes, void *stream);
int fp5_dequantize(const void *hi_plane, const void *lo_plane, const uint16_t *scales,
                   int64_t N, int64_t K, uint16_t *W_hat, void *stream);
size_t fp5_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int split_k);
int fp5_linear(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
               const uint16_t *scales, int64_t N, int64_t K, uint16_t *Y,
               void *workspace, size_t workspace_bytes, void *stream, int variant, int split_k);

/*
 * FP6 in plane layout 2: the same codes, scales and sizes (N*K/2 + N*K/4 bytes), with the bits of
 * the two planes placed so that a few logic operations merge them into the densely packed six-bit
 * string that gfx950's packed E3M2 -> fp16 conversion (v_cvt_scalef32_pk32_f16_bf6) consumes - a
 * hardware alternative to the bit padding of Section 5.2 that keeps the 4+2 split of Section 5.1
 * (the 4-bit plane still holds sign and exponent bits only, the 2-bit plane mantissa bits only).
 * Tiles, tile order, lanes and fragments are those of layout 1.  A "unit" is the 32 weights a lane
 * holds for one 32-wide k block of a tile (kk/32 = q): element i = 8t + e, where t = nn/16 is the
 * 16-channel fragment and e = kk%8.  Let STR be the 192-bit string with the code of element i
 * (s eee mm) at bits 6i .. 6i+5, and STR[j] its dword j.  Bit p of STR[j] is a mantissa bit iff
 * (32j + p) % 6 < 2.  The lane's dwords in the planes are
 *   2-bit plane, byte offset ti*1024 + l*16 + 8q:      B0, B1
 *   4-bit plane, byte offset ti*2048 + q*1024 + l*16:  A0, A1, A2, A3
 * with, writing SE(j) for the sign/exponent positions of STR[j] and MA(j) for its mantissa positions,
 *   B0 = STR[0]&MA(0) | STR[1]&MA(1) | STR[2]&MA(2)        B1 = the same of STR[3], STR[4], STR[5]
 *   A0 = STR[0]&SE(0) | STR[4]&MA(0)
 *   A1 = STR[1]&SE(1) | (STR[4] & 0x0C30C30C) << 2
 *   A2 = STR[2]&SE(2) | (STR[5] & 0x030C30C3) << 2
 *   A3 = STR[3]&SE(0) | rotate_left(STR[5] & 0xF0C30C30, 2)
 * (SE(0) = SE(3) = 0x3CF3CF3C, SE(1) = SE(4) = 0xCF3CF3CF, SE(2) = SE(5) = 0xF3CF3CF3, MA = ~SE.)
 * The result of the linear layer is the same up to fp32 summation order: the converted operands
 * are the FP6 values themselves and the row scale is applied without the 2^12.  Calls mirror the
 * layout-1 ones (row-wise scales; no tuning hints besides block_m).
 */
int fp6_quantize_pack_v2(const uint16_t *W, int64_t N, int64_t K, void *hi_plane, void *lo_plane,
                         uint16_t *scales, void *stream);
int fp6_unpack_codes_v2(const void *hi_plane, const void *lo_plane, int64_t N, int64_t K,
                        uint8_t *codes, void *stream);
int fp6_dequantize_v2(const void *hi_plane, const void *lo_plane, const uint16_t *scales,
                      int64_t N, int64_t K, uint16_t *W_hat, void *stream);
size_t fp6_linear_v2_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int split_k);
int fp6_linear_v2(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
                  const uint16_t *scales, int64_t N, int64_t K, uint16_t *Y,
                  void *workspace, size_t workspace_bytes, void *stream, int variant, int split_k);

/*
 * bf16 activations (Section 2 allows FP16 or BF16 around the FP6 weights): X and Y hold bf16 bit
 * patterns, everything else is as in fp6_linear_v2 - the planes of layout 2, fp16 row scales, fp32
 * accumulation, the same workspace size (fp6_linear_v2_workspace_bytes) and the same plans.  The
 * weights reach the matrix cores through the bf16 form of the hardware conversion, which is exact
 * for every E3M2 code; Y[m][n] = bf16_RNE(S_n * sum_k X[m][k] * v(c[n][k])) up to fp32 summation
 * order.  (Bit padding as in Section 5.2 does not carry over: padded into bf16 the weights would be
 * scaled by 2^-124 and their products would leave the normal range of the fp32 accumulator.)
 */
int fp6_linear_v2_bf16(const uint16_t *X, int64_t M, const void *hi_plane, const void *lo_plane,
                       const uint16_t *scales, int64_t N, int64_t K, uint16_t *Y,
                       void *workspace, size_t workspace_bytes, void *stream, int variant, int split_k);

/*
 * Measurement aids (no passage of the paper: they measure the chip, not the method).  Each
 * launches one kernel on `stream` and returns at once, like the calls above.
 *   fp6_probe_read: `workgroups` workgroups of 256 lanes stream `bytes` (rounded down to 16) from
 *     `buf` (device, 16-byte aligned) with 128-bit non-temporal loads; `sink` (device, at least
 *     16 * workgroups bytes) receives one folded word per wavefront.  bytes / duration is the read
 *     rate a kernel that does nothing else reaches on this chip.
 *   fp6_probe_mfma: `workgroups` workgroups of 4 wavefronts; each wavefront issues 8 * iters
 *     MFMAs on 8 independent accumulators; 4 + 2 operand fragments held in registers,
 *     pseudo-random fp16 in (-1, 1) if random_operands != 0, else zeros.  `form`:
 *     0 = v_mfma_f32_16x16x32_f16; 1 = v_mfma_f32_32x32x16_f16; 2 = form 0 with two independent
 *     integer vector instructions behind every MFMA (the instruction mix of the tiled kernel's
 *     loop, whose unpack shares the vector issue port with the MFMAs).  `sink` (device, at least
 *     1024 * workgroups bytes) receives one float per lane.  Work of a launch:
 *     workgroups * 4 * 8 * iters * 16384 flop, twice that for form 1.
 * Errors: FP6_ERR_NULL, FP6_ERR_ALIGN, FP6_ERR_SHAPE (sizes out of range: workgroups 1 .. 2^20,
 * iters 1 .. 2^24, bytes >= 16), FP6_ERR_VARIANT (form), FP6_ERR_WORKSPACE (sink too small),
 * FP6_ERR_HIP.
 */
int fp6_probe_read(const void *buf, size_t bytes, int workgroups, void *sink, size_t sink_bytes,
                   void *stream);
int fp6_probe_mfma(int workgroups, int iters, int random_operands, int form, void *sink,
                   size_t sink_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FP6_LINEAR_H */
