// Tiled kernel (any M) of the W6A16 linear layer for gfx950.
//
// A workgroup of four wavefronts computes a BM x 256 block of Y.  The wavefronts stand
// side by side along N (64 output channels each), so every packed weight is fetched and
// padded to fp16 (bias shift, Section 5.2) by exactly one wavefront, straight from its
// three 128-bit plane loads into MFMA operand registers - the dequantized weight never
// touches LDS.  Only the activations are shared: the BM x 64 slice of X for a k tile
// goes from global memory directly into LDS (global_load_lds, no register staging)
// into a ring of D stages, and is read by all four wavefronts as MFMA operands.  Rows
// are not padded; the 16-byte chunk c of row r is stored at chunk position c ^ (r & 7),
// which makes both the DMA writes and the 128-bit operand reads bank-conflict free.
// The plane loads of the wavefront run D-1 tiles ahead in a register ring.  The row
// scale is applied once, after the accumulation (Section 5.2).  K may be split over
// workgroups; the slices meet in an fp32 workspace exactly as in the decode kernel.
#include "fp6_common.hpp"
#include "fp6_internal.hpp"
#include "fp6_reduce.hpp"

namespace fp6 {

#define FP6_GLOBAL_AS __attribute__((address_space(1)))
#define FP6_LDS_AS __attribute__((address_space(3)))

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

template <int BM, int D>
__global__ __launch_bounds__(256, 2) void gemm_kernel(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, int split_k)
{
    constexpr int MT = BM / 16;            // 16-row blocks of X per workgroup
    constexpr int XL = BM / 32;            // 1 KB DMA loads of X per wavefront and k tile
    constexpr int kLoads = XL + 3;         // vector-memory loads per wavefront and k tile
    constexpr int kStageHalfs = BM * kTile;
    __shared__ __align__(16) uint16_t xs[D][kStageHalfs];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ktiles = K / kTile, nblocks = N / kTile;
    const int mblk = (M + BM - 1) / BM;
    int id = blockIdx.x;
    const int s = id % split_k;
    id /= split_k;
    const int mb = id % mblk, nbw = id / mblk;
    const int kt_per = ktiles / split_k;
    const int kt_begin = s * kt_per, kt_end = kt_begin + kt_per;
    const int m0 = mb * BM;
    const int nb = nbw * 4 + wave;
    const bool wvalid = nb < nblocks;
    const size_t tile0 = (size_t)(wvalid ? nb : 0) * ktiles;
    const int i = lane & 15, g = lane >> 4;

    // DMA of the X slice: wavefront w moves the 8-row groups j = w*XL .. w*XL+XL-1; lane l
    // of a group fetches row 8j + l/8, chunk (l%8) ^ (l/8), and lands at chunk position l%8.
    const uint16_t* xsrc[XL];
#pragma unroll
    for (int p = 0; p < XL; p++) {
        int row = m0 + (wave * XL + p) * 8 + (lane >> 3);
        row = row < M ? row : M - 1;      // rows past M are computed on valid data and dropped
        xsrc[p] = X + (size_t)row * K + (((lane & 7) ^ (lane >> 3)) * 8);
    }
    // operand reads: row r = 16a + i, chunk 4q + g, at position (4q + g) ^ (i & 7)
    const int xoff0 = i * kTile + ((g ^ (i & 7)) * 8);
    const int xoff1 = i * kTile + (((4 + g) ^ (i & 7)) * 8);

    float4v acc[MT][4];
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
        for (int t = 0; t < 4; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};

    TileRaw raw[D];

    // every call issues exactly kLoads vector-memory loads per wavefront
    auto issue = [&](int kt, int stage, TileRaw& dst) {
#pragma unroll
        for (int p = 0; p < XL; p++)
            __builtin_amdgcn_global_load_lds((const FP6_GLOBAL_AS void*)(xsrc[p] + (size_t)kt * kTile),
                                             (FP6_LDS_AS void*)&xs[stage][(wave * XL + p) * 512], 16, 0, 0);
        dst = load_tile(hi, lo, tile0 + kt, lane);
    };

#pragma unroll
    for (int u = 0; u < D - 1; u++) issue(min(kt_begin + u, kt_end - 1), u, raw[u]);

    for (int kt = kt_begin; kt < kt_end; kt += D) {
#pragma unroll
        for (int u = 0; u < D; u++) {
            if (kt + u < kt_end) {
                // the loads of this k tile were issued D-1 steps ago; D-2 younger groups may stay in flight
                wait_vmcnt<(D - 2) * kLoads>();
                __syncthreads();          // everyone's DMA landed; everyone is done with the stage refilled next
                issue(min(kt + u + D - 1, kt_end - 1), (u + D - 1) % D, raw[(u + D - 1) % D]);
                const uint16_t* xst = xs[u];
#pragma unroll
                for (int q = 0; q < 2; q++) {
                    half8 xf[MT];
#pragma unroll
                    for (int a = 0; a < MT; a++)
                        xf[a] = *reinterpret_cast<const half8*>(xst + a * 16 * kTile + (q ? xoff1 : xoff0));
#pragma unroll
                    for (int t = 0; t < 4; t++) {
                        half8 w = unpack_tile_fragment(raw[u], 2 * t + q);
#pragma unroll
                        for (int a = 0; a < MT; a++) acc[a][t] = mfma16x16x32(w, xf[a], acc[a][t]);
                    }
                }
            }
        }
    }
    wait_vmcnt<0>();     // the over-fetched ring slots must land before LDS is given back

    // ---- K-slices of other workgroups
    if (split_k > 1) {
        const int tile = nbw * mblk + mb, ntiles = gridDim.x / split_k;
        constexpr uint32_t kTileBytes = MT * 4 * 256 * 16;
        if (wvalid) {
            __amdgpu_buffer_rsrc_t win = partial_window(partials + ((size_t)s * ntiles + tile) * (MT * 4 * 256), kTileBytes);
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < 4; t++) store_partial(win, (a * 4 + t) * 256 + tid, acc[a][t]);
        }
        if (!arrive_last(&counters[tile], (uint32_t)split_k)) return;
        if (wvalid) {
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < 4; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
            for (int ss = 0; ss < split_k; ss++) {
                __amdgpu_buffer_rsrc_t win =
                    partial_window(partials + ((size_t)ss * ntiles + tile) * (MT * 4 * 256), kTileBytes);
#pragma unroll
                for (int a = 0; a < MT; a++)
#pragma unroll
                    for (int t = 0; t < 4; t++) acc[a][t] += load_partial(win, (a * 4 + t) * 256 + tid);
            }
        }
    }

    // ---- epilogue: lane holds rows n = 16t + 4g + r of column m = 16a + i
    if (!wvalid) return;
    float sc[4][4];
#pragma unroll
    for (int t = 0; t < 4; t++) {
        const half4 h = *reinterpret_cast<const half4*>(scales + (size_t)nb * kTile + t * 16 + g * 4);
#pragma unroll
        for (int r = 0; r < 4; r++) sc[t][r] = (float)h[r] * 4096.0f;
    }
#pragma unroll
    for (int a = 0; a < MT; a++) {
        const int m = m0 + a * 16 + i;
        if (m < M) {
#pragma unroll
            for (int t = 0; t < 4; t++) {
                half4 y;
#pragma unroll
                for (int r = 0; r < 4; r++) y[r] = (_Float16)(acc[a][t][r] * sc[t][r]);
                *reinterpret_cast<half4*>(Y + (size_t)m * N + (size_t)nb * kTile + t * 16 + g * 4) = y;
            }
        }
    }
}

template <int BM, int D>
static hipError_t launch_gemm_t(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                                const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                                hipStream_t stream)
{
    uint32_t* counters = reinterpret_cast<uint32_t*>(workspace);
    float4v* partials = reinterpret_cast<float4v*>(reinterpret_cast<char*>(workspace) + kCounterBytes);
    const int64_t mblk = (M + BM - 1) / BM, nblk = (N / kTile + 3) / 4;
    const unsigned grid = (unsigned)(mblk * nblk * p.split_k);
    hipLaunchKernelGGL((gemm_kernel<BM, D>), dim3(grid), dim3(256), 0, stream, X, (int)M, (const u32x4*)hi,
                       (const u32x4*)lo, scales, (int)N, (int)K, Y, partials, counters, p.split_k);
    return hipGetLastError();
}

hipError_t launch_gemm(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                       hipStream_t stream)
{
    switch (p.block_m * 10 + p.depth) {
        case 323: return launch_gemm_t<32, 3>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 324: return launch_gemm_t<32, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 643: return launch_gemm_t<64, 3>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 644: return launch_gemm_t<64, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 1283: return launch_gemm_t<128, 3>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        default: return launch_gemm_t<128, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
}

}  // namespace fp6
