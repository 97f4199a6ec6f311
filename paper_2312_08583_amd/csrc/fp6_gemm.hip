// Tiled kernel (any M) of the W6A16 linear layer for gfx950.
//
// A workgroup of eight wavefronts (two per SIMD) computes a BM x 512 block of Y.  The
// wavefronts stand side by side along N (64 output channels each), so every packed
// weight is fetched and padded to fp16 (bias shift, Section 5.2) by exactly one
// wavefront of the workgroup and goes straight into MFMA operand registers - the
// dequantized weight never exists in memory.  Only the activations are shared.
//
// All global traffic of the main loop is asynchronous DMA into LDS (global_load_lds,
// 16 bytes per lane, no register staging), into a ring of D stages per workgroup:
//   - the BM x 64 slice of X for a k tile (read by all eight wavefronts as MFMA
//     operands).  Rows are not padded; the 16-byte chunk c of row r is stored at chunk
//     position c ^ (r & 7), which keeps the DMA writes and the 128-bit operand reads
//     free of bank conflicts;
//   - each wavefront's own 3 KB of packed planes for that k tile (lane-linear, exactly
//     the order the planes have in memory).
// The DMA is issued from inline assembly and waited for with explicit s_waitcnt vmcnt:
// every step issues the same number of loads per wavefront, so "at most (D-2) groups
// still in flight" is a constant, and the compiler (which cannot see these loads) has
// no reason to drain the queue.  One barrier per k tile publishes the landed stage and
// frees the stage consumed in the previous step.  The row scale is applied once, after
// the accumulation (Section 5.2).  K may be split over workgroups; the slices meet in
// an fp32 workspace exactly as in the decode kernel.
#include "fp6_common.hpp"
#include "fp6_internal.hpp"
#include "fp6_reduce.hpp"

namespace fp6 {

constexpr int kGemmWaves = 8;
constexpr int kWaveTileBytes = kHiTileBytes + kLoTileBytes;   // 3072: one wavefront's planes of one tile

// 16 bytes per lane from (base + lane_offset) to LDS address lds + 16 * lane (lds is wave-uniform).
// M0 carries the LDS address; nothing else in these kernels uses M0 (gfx9 DS instructions do not),
// and the compiler does not accept it in a clobber list.
__device__ __forceinline__ void dma16(const void* base, uint32_t lane_offset, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(base), "s"(lds)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

template <int BM, int D>
__global__ __launch_bounds__(kGemmWaves * 64) void gemm_kernel(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, int split_k)
{
    constexpr int MT = BM / 16;                         // 16-row blocks of X per workgroup
    constexpr int XG = BM / 8;                          // 8-row groups (1 KB of DMA each) per stage
    constexpr int XL = XG >= kGemmWaves ? XG / kGemmWaves : 1;   // X groups moved per wavefront and k tile
    constexpr int kLoads = XL + 3;                      // DMA instructions per wavefront and k tile
    constexpr int kXBytes = BM * kTile * 2;
    constexpr int kStageBytes = kXBytes + kGemmWaves * kWaveTileBytes;
    __shared__ __align__(16) unsigned char smem[D * kStageBytes];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ktiles = K / kTile, nblocks = N / kTile;
    const int mblk = (M + BM - 1) / BM;
    int id = blockIdx.x;
    const int s = id % split_k;
    id /= split_k;
    const int mb = id % mblk, nbw = id / mblk;
    const int kt_per = ktiles / split_k;
    const int kt_begin = s * kt_per, kt_end = kt_begin + kt_per;
    const int m0 = mb * BM;
    const int nb = nbw * kGemmWaves + wave;
    const bool wvalid = nb < nblocks;
    const size_t tile0 = (size_t)(wvalid ? nb : 0) * ktiles;
    const int i = lane & 15, g = lane >> 4;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    // X DMA: this wavefront moves the 8-row groups j = (wave*XL + p) % XG; lane l of a group
    // fetches row 8j + l/8, chunk (l%8) ^ (l/8), and lands at chunk position l%8.
    uint32_t xlane[XL], xlds[XL];
#pragma unroll
    for (int p = 0; p < XL; p++) {
        const int j = (wave * XL + p) % XG;
        int row = m0 + j * 8 + (lane >> 3);
        row = row < M ? row : M - 1;      // rows past M are computed on valid data and dropped
        xlane[p] = (uint32_t)row * (uint32_t)K * 2u + (uint32_t)(((lane & 7) ^ (lane >> 3)) * 16);
        xlds[p] = j * 1024;
    }
    const uint32_t wlane = lane * 16;
    const uint32_t wlds = kXBytes + wave * kWaveTileBytes;

    // kLoads DMA instructions per call, always
    auto issue = [&](int kt, int stage) {
        const uint32_t sb = smem_base + stage * kStageBytes;
        const unsigned char* xb = reinterpret_cast<const unsigned char*>(X) + (size_t)kt * (kTile * 2);
#pragma unroll
        for (int p = 0; p < XL; p++) dma16(xb, xlane[p], sb + xlds[p]);
        const unsigned char* hb = reinterpret_cast<const unsigned char*>(hi) + (tile0 + kt) * kHiTileBytes;
        const unsigned char* lb = reinterpret_cast<const unsigned char*>(lo) + (tile0 + kt) * kLoTileBytes;
        dma16(hb, wlane, sb + wlds);
        dma16(hb + 1024, wlane, sb + wlds + 1024);
        dma16(lb, wlane, sb + wlds + 2048);
    };

    // operand reads: row r = 16a + i, chunk 4q + g, at position (4q + g) ^ (i & 7)
    const int xoff0 = i * (kTile * 2) + ((g ^ (i & 7)) * 16);
    const int xoff1 = i * (kTile * 2) + (((4 + g) ^ (i & 7)) * 16);

    float4v acc[MT][4];
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
        for (int t = 0; t < 4; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int u = 0; u < D - 1; u++) issue(min(kt_begin + u, kt_end - 1), u);

    // one k tile: its DMA was issued D-1 steps ago; D-2 younger groups may stay in flight
    auto step = [&](int kt, int u) {
        wait_vmcnt<(D - 2) * kLoads>();
        __syncthreads();          // everyone's DMA landed; everyone is done with the stage refilled next
        issue(min(kt + D - 1, kt_end - 1), (u + D - 1) % D);
        const unsigned char* st = smem + u * kStageBytes;
        TileRaw raw;
        raw.hi0 = *reinterpret_cast<const u32x4*>(st + wlds + wlane);
        raw.hi1 = *reinterpret_cast<const u32x4*>(st + wlds + 1024 + wlane);
        raw.lo = *reinterpret_cast<const u32x4*>(st + wlds + 2048 + wlane);
#pragma unroll
        for (int q = 0; q < 2; q++) {
            half8 xf[MT];
#pragma unroll
            for (int a = 0; a < MT; a++)
                xf[a] = *reinterpret_cast<const half8*>(st + a * 16 * (kTile * 2) + (q ? xoff1 : xoff0));
#pragma unroll
            for (int t = 0; t < 4; t++) {
                half8 w = unpack_tile_fragment(raw, 2 * t + q);
#pragma unroll
                for (int a = 0; a < MT; a++) acc[a][t] = mfma16x16x32(w, xf[a], acc[a][t]);
            }
        }
    };

    int kt = kt_begin;
    for (; kt + D <= kt_end; kt += D) {      // steady state: branch-free trips of D tiles
#pragma unroll
        for (int u = 0; u < D; u++) step(kt + u, u);
    }
#pragma unroll
    for (int u = 0; u < D - 1; u++) {        // the last (kt_end - kt_begin) % D tiles
        if (kt + u < kt_end) step(kt + u, u);
    }
    wait_vmcnt<0>();     // the over-fetched ring slots must land before LDS is given back
    __syncthreads();

    // ---- K-slices of other workgroups
    if (split_k > 1) {
        const int tile = nbw * mblk + mb, ntiles = gridDim.x / split_k;
        constexpr int kTileRegs = MT * 4 * kGemmWaves * 64;      // float4 per output tile
        if (wvalid) {
            __amdgpu_buffer_rsrc_t win = partial_window(partials + ((size_t)s * ntiles + tile) * kTileRegs, kTileRegs * 16);
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < 4; t++) store_partial(win, (a * 4 + t) * (kGemmWaves * 64) + tid, acc[a][t]);
        }
        if (!arrive_last(&counters[tile], (uint32_t)split_k)) return;
        if (wvalid) {
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < 4; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
            for (int ss = 0; ss < split_k; ss++) {
                __amdgpu_buffer_rsrc_t win = partial_window(partials + ((size_t)ss * ntiles + tile) * kTileRegs, kTileRegs * 16);
#pragma unroll
                for (int a = 0; a < MT; a++)
#pragma unroll
                    for (int t = 0; t < 4; t++) acc[a][t] += load_partial(win, (a * 4 + t) * (kGemmWaves * 64) + tid);
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
    const int64_t mblk = (M + BM - 1) / BM, nblk = (N / kTile + kGemmWaves - 1) / kGemmWaves;
    const unsigned grid = (unsigned)(mblk * nblk * p.split_k);
    hipLaunchKernelGGL((gemm_kernel<BM, D>), dim3(grid), dim3(kGemmWaves * 64), 0, stream, X, (int)M, (const u32x4*)hi,
                       (const u32x4*)lo, scales, (int)N, (int)K, Y, partials, counters, p.split_k);
    return hipGetLastError();
}

hipError_t launch_gemm(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                       hipStream_t stream)
{
    switch (p.block_m) {
        case 32: return launch_gemm_t<32, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 64: return launch_gemm_t<64, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        default: return launch_gemm_t<128, 3>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
}

}  // namespace fp6
