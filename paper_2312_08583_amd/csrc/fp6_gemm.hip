// Tiled kernel (any M) of the W6A16 linear layer for gfx950.
//
// A workgroup of four wavefronts computes a BM x 256 block of Y.  The wavefronts stand
// side by side along N (64 output channels each), so every packed weight is fetched and
// padded to fp16 (bias shift, Section 5.2) by exactly one wavefront, straight from its
// three 128-bit plane loads into MFMA operand registers - the dequantized weight never
// touches LDS.  Only the activations are shared: the BM x 64 slice of X for the current
// k tile is staged in LDS (double buffered, rows padded by 16 bytes so that the 128-bit
// operand reads are bank-conflict free) and read by all four wavefronts.  The row scale
// is applied once, after the accumulation (Section 5.2).  K may be split over
// workgroups; the slices meet in an fp32 workspace exactly as in the decode kernel.
#include "fp6_common.hpp"
#include "fp6_internal.hpp"
#include "fp6_reduce.hpp"

namespace fp6 {

constexpr int kLdsRow = kTile + 8;   // halfs per staged row of X (64 + 16 bytes of padding)

template <int BM>
__global__ __launch_bounds__(256) void gemm_kernel(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, int split_k)
{
    constexpr int MT = BM / 16;        // 16-row blocks of X per workgroup
    constexpr int XL = BM / 32;        // 16-byte loads of X per thread and k tile
    __shared__ __align__(16) uint16_t xs[2][BM][kLdsRow];

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

    // this thread's share of the X slice: rows xr + 32p, 16-byte column xc
    const int xr = tid >> 3, xc = tid & 7;
    const uint16_t* xsrc[XL];
#pragma unroll
    for (int p = 0; p < XL; p++) {
        int row = m0 + xr + 32 * p;
        row = row < M ? row : M - 1;      // rows past M are computed on valid data and dropped
        xsrc[p] = X + (size_t)row * K + xc * 8;
    }

    float4v acc[MT][4];
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
        for (int t = 0; t < 4; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};

    uint4 xg[XL];
    TileRaw cur, nxt;
#pragma unroll
    for (int p = 0; p < XL; p++) xg[p] = *reinterpret_cast<const uint4*>(xsrc[p] + (size_t)kt_begin * kTile);
    cur = load_tile(hi, lo, tile0 + kt_begin, lane);
#pragma unroll
    for (int p = 0; p < XL; p++) *reinterpret_cast<uint4*>(&xs[0][xr + 32 * p][xc * 8]) = xg[p];
    __syncthreads();

    int buf = 0;
    for (int kt = kt_begin; kt < kt_end; kt++) {
        const bool more = kt + 1 < kt_end;
        if (more) {
#pragma unroll
            for (int p = 0; p < XL; p++) xg[p] = *reinterpret_cast<const uint4*>(xsrc[p] + (size_t)(kt + 1) * kTile);
            nxt = load_tile(hi, lo, tile0 + kt + 1, lane);
        }
#pragma unroll
        for (int q = 0; q < 2; q++) {
            half8 xf[MT];
#pragma unroll
            for (int a = 0; a < MT; a++)
                xf[a] = *reinterpret_cast<const half8*>(&xs[buf][a * 16 + i][q * 32 + g * 8]);
#pragma unroll
            for (int t = 0; t < 4; t++) {
                half8 w = unpack_tile_fragment(cur, 2 * t + q);
#pragma unroll
                for (int a = 0; a < MT; a++) acc[a][t] = mfma16x16x32(w, xf[a], acc[a][t]);
            }
        }
        if (more) {
#pragma unroll
            for (int p = 0; p < XL; p++) *reinterpret_cast<uint4*>(&xs[buf ^ 1][xr + 32 * p][xc * 8]) = xg[p];
        }
        __syncthreads();
        cur = nxt;
        buf ^= 1;
    }

    // ---- K-slices of other workgroups
    if (split_k > 1) {
        const int tile = nbw * mblk + mb, ntiles = gridDim.x / split_k;
        if (wvalid) {
            float4v* dst = partials + ((size_t)s * ntiles + tile) * (MT * 4 * 256) + tid;
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < 4; t++) dst[(a * 4 + t) * 256] = acc[a][t];
        }
        if (!arrive_last(&counters[tile], (uint32_t)split_k)) return;
        if (wvalid) {
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < 4; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
            for (int ss = 0; ss < split_k; ss++) {
                const float4v* src = partials + ((size_t)ss * ntiles + tile) * (MT * 4 * 256) + tid;
#pragma unroll
                for (int a = 0; a < MT; a++)
#pragma unroll
                    for (int t = 0; t < 4; t++) acc[a][t] += load_partial(&src[(a * 4 + t) * 256]);
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

template <int BM>
static hipError_t launch_gemm_t(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                                const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                                hipStream_t stream)
{
    uint32_t* counters = reinterpret_cast<uint32_t*>(workspace);
    float4v* partials = reinterpret_cast<float4v*>(reinterpret_cast<char*>(workspace) + kCounterBytes);
    const int64_t mblk = (M + BM - 1) / BM, nblk = (N / kTile + 3) / 4;
    const unsigned grid = (unsigned)(mblk * nblk * p.split_k);
    hipLaunchKernelGGL((gemm_kernel<BM>), dim3(grid), dim3(256), 0, stream, X, (int)M, (const u32x4*)hi,
                       (const u32x4*)lo, scales, (int)N, (int)K, Y, partials, counters, p.split_k);
    return hipGetLastError();
}

hipError_t launch_gemm(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                       hipStream_t stream)
{
    switch (p.block_m) {
        case 32: return launch_gemm_t<32>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 64: return launch_gemm_t<64>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        default: return launch_gemm_t<128>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
}

}  // namespace fp6
