// Tiled kernel: dispatch, and the instantiations of the method itself (FP6, bias-shift unpack, row scales).
#include "fp6_gemm_kernel.hpp"

namespace fp6 {

hipError_t launch_gemm(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                       hipStream_t stream)
{
    if (p.format != kE3M2 || p.gshift >= 0 || p.dequant != kBiasShift)
        return launch_gemm_variant(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    // (The kernel template also supports four wavefronts owning 128 channels each, WN = 2; that shape
    // measured slower at every block size and is not instantiated.)
    // Four-wavefront workgroups are built so that two fit a compute unit (at most 256 registers per lane and
    // 80 KB of LDS: a ring of 4, 3 and 2 stages at 32, 64 and 128 rows), i.e. two wavefronts per SIMD as with
    // eight-wavefront workgroups; measured 4-10 % faster than deeper rings with one workgroup per unit.
    // Two K-ways inside a workgroup of 128 x 256: eight wavefronts, a ring of two stages for the activations (two k
    // tiles each) and three for the planes: 136 KB of LDS.
    if (p.gbn == 4 && p.kw == 2)
        return launch_gemm_t<128, 3, 1, kBiasShift, false, kE3M2, 4, 2, 2>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.gbn == 4) {
        switch (p.block_m) {
            case 32: return launch_gemm_t<32, 4, 1, kBiasShift, false, kE3M2, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
            case 64: return launch_gemm_t<64, 3, 1, kBiasShift, false, kE3M2, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
            default: return launch_gemm_t<128, 2, 1, kBiasShift, false, kE3M2, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        }
    }
    switch (p.block_m) {
        case 32: return launch_gemm_t<32, 4, 1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 64: return launch_gemm_t<64, 4, 1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        default: return launch_gemm_t<128, 3, 1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
}

}  // namespace fp6
