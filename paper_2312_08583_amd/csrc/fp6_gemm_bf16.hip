// Tiled kernel: the instantiations for bf16 activations (plane layout 2, hardware conversion to bf16).
#include "fp6_gemm_kernel.hpp"

namespace fp6 {

hipError_t launch_gemm_bf16(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                            const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                            hipStream_t stream)
{
    if (p.gbn == 4) {
        if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M2B, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        if (p.block_m == 64) return launch_gemm_t<64, 3, 1, kBiasShift, false, kE3M2B, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_gemm_t<128, 2, 1, kBiasShift, false, kE3M2B, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.block_m == 32) return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M2B>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.block_m == 64) return launch_gemm_t<64, 4, 1, kBiasShift, false, kE3M2B>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    return launch_gemm_t<128, 3, 1, kBiasShift, false, kE3M2B>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
}

}  // namespace fp6
