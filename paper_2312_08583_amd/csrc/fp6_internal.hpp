// Host-side declarations shared by the translation units of the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/fp6_linear.h"

namespace fp6 {

// Weight formats.  kE3M2: FP6, planes of 4 + 2 bits (Section 5.1).  kE3M1: FP5, the same
// sign/exponent plane plus a 1-bit mantissa plane ("4+1"; Section 4, Section 6).
// kE3M2H: FP6 again, with the bits of the two planes placed so that they merge into the densely packed
// six-bit string that gfx950's packed E3M2 -> fp16 conversion instruction consumes (plane layout 2).
// kE3M2B: the planes of kE3M2H with bf16 activations and bf16 output (the conversion to bf16 is the same instruction's
//         bf16 form; plain bit padding does not carry over to bf16, whose padded values would sit at 2^-124).
enum Format { kE3M2 = 6, kE3M1 = 5, kE3M2H = 7, kE3M2B = 8 };
constexpr bool layout2(int format) { return format == kE3M2H || format == kE3M2B; }

// Workspace layout: [arrival counters: kCounterBytes][meeting slots: kSlotBytes][fp32 partial sums].
// The first two regions (kZeroBytes) are zero whenever no call is running.
constexpr int kCounterStride = 16;      // uint32 words between two counters: one 64-byte line each, so that
                                        // arrivals at different tiles do not queue up behind one another
constexpr int kMaxCounters = 1024;
constexpr size_t kCounterBytes = (size_t)kMaxCounters * kCounterStride * sizeof(uint32_t);
constexpr size_t kSlotBytes = (size_t)4 << 20;
constexpr size_t kZeroBytes = kCounterBytes + kSlotBytes;

// `format` = 6 (E3M2) or 5 (E3M1).  `block` = elements along K that share a scale (K itself for the row-wise scheme); scale (n, g) at scales[g*N + n]
hipError_t launch_quantize_pack(int format, const uint16_t* W, int64_t N, int64_t K, int64_t block, void* hi, void* lo,
                                uint16_t* scales, hipStream_t stream);
hipError_t launch_unpack_codes(int format, const void* hi, const void* lo, int64_t N, int64_t K, uint8_t* codes,
                               hipStream_t stream);
hipError_t launch_dequantize(int format, const void* hi, const void* lo, const uint16_t* scales, int64_t N, int64_t K,
                             int64_t block, uint16_t* W_hat, hipStream_t stream);

// A fully resolved launch plan for fp6_linear.
struct LinearPlan {
    int variant;        // FP6_VARIANT_DECODE or FP6_VARIANT_GEMM
    int split_k;        // K-slices handled by separate workgroups (>= 1)
    int block_m;        // GEMM: rows of X per workgroup (32, 64 or 128); DECODE: 16
    int waves;          // wavefronts per workgroup
    int depth;          // tiles in the per-wavefront prefetch ring
    size_t partial_bytes;   // fp32 partial sums needed in the workspace (0 if split_k == 1)
    int counters;       // arrival counters used (0 if split_k == 1)
    int format;         // 6: FP6 E3M2 (4+2 planes); 5: FP5 E3M1 (4+1 planes)
    int gshift;         // fine-grained scales: log2(block / 64); -1 = one scale per row
    int dequant;        // 0: bias-shift unpack (the method); 1, 2: ablations (integer re-bias, fp16 multiply)
    int gbn;            // GEMM: 64-channel blocks (= wavefronts) per workgroup: 8 or 4
    int half_tiles;     // DECODE: workgroups own 32 channels (half a tile) instead of 64
    int pairwise;       // DECODE with split_k > 1: K-slices meet pairwise in the slot region (1) or at a counter (0)
    int kw;             // GEMM: K-ways inside the workgroup (1, or 2 with gbn = 4 and block_m = 128)
};

// Heuristic (or caller-forced) plan; returns false if the request is invalid for the shape.
// `block` = elements along K per scale (0 = row-wise).
bool make_plan(int format, int64_t M, int64_t N, int64_t K, int64_t block, int variant, int split_k, LinearPlan* plan);

// One layer of a group of layers launched together (fp6_linear_group).
struct GroupLayer {
    const uint16_t* X;
    const void* hi;
    const void* lo;
    const uint16_t* scales;
    uint16_t* Y;
    int64_t N;
};
hipError_t launch_decode_group(const LinearPlan& p, int count, const GroupLayer* layers, int64_t M, int64_t K, void* workspace,
                               hipStream_t stream);

hipError_t launch_decode(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                         const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                         hipStream_t stream);
// fp6_gemm_variants.hip: plans with an ablation unpack, fine-grained scales or the five-bit format
hipError_t launch_gemm_variant(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                               const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                               hipStream_t stream);
hipError_t launch_gemm_bf16(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                               const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                               hipStream_t stream);
hipError_t launch_gemm(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                       hipStream_t stream);

}  // namespace fp6
