// Tiled kernel: the instantiations beside the method itself - bias-shift ablations, fine-grained scales, FP5.
#include "fp6_gemm_kernel.hpp"

namespace fp6 {

hipError_t launch_gemm_variant(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                               const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                               hipStream_t stream)
{
    if (p.format == kE3M2B) return launch_gemm_bf16(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.format == kE3M2H && p.gbn == 4) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M2H, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        if (p.block_m == 64) return launch_gemm_t<64, 3, 1, kBiasShift, false, kE3M2H, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<128, 2, 1, kBiasShift, false, kE3M2H, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.format == kE3M2H) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M2H>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        if (p.block_m == 64) return launch_gemm_t<64, 4, 1, kBiasShift, false, kE3M2H>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<128, 3, 1, kBiasShift, false, kE3M2H>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.format == kE3M1 && p.gbn == 4) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M1, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        if (p.block_m == 64) return launch_gemm_t<64, 3, 1, kBiasShift, false, kE3M1, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<128, 2, 1, kBiasShift, false, kE3M1, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.format == kE3M1) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        if (p.block_m == 64) return launch_gemm_t<64, 4, 1, kBiasShift, false, kE3M1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<128, 3, 1, kBiasShift, false, kE3M1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.gshift >= 0 && p.gbn == 4) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, true, kE3M2, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<64, 3, 1, kBiasShift, true, kE3M2, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.gshift >= 0) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, true>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<64, 4, 1, kBiasShift, true>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    switch (p.block_m + p.dequant * 1000) {
        case 1032: return launch_gemm_t<32, 4, 1, kIntRebias>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 1064: return launch_gemm_t<64, 4, 1, kIntRebias>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 1128: return launch_gemm_t<128, 3, 1, kIntRebias>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 2032: return launch_gemm_t<32, 4, 1, kHalfMul>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 2064: return launch_gemm_t<64, 4, 1, kHalfMul>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        default: return launch_gemm_t<128, 3, 1, kHalfMul>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
}

}  // namespace fp6
