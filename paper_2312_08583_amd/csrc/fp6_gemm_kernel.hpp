// Tiled kernel (any M) of the W6A16 linear layer for gfx950: the kernel template and its launcher.
// Included by the translation units that instantiate it (fp6_gemm.hip: the FP6 bias-shift kernels;
// fp6_gemm_variants.hip: ablations, fine-grained scales, FP5).
//
// A workgroup computes a BM x (64 * GBN) block of Y, GBN = 8 or 4.  Its wavefronts stand side by
// side along N, each owning WN 64-wide blocks of output channels (WN = 1 in every instantiated
// kernel: one wavefront per 64 channels, two per SIMD at GBN = 8).  Every packed
// weight is fetched and padded to fp16 (bias shift, Section 5.2) by exactly one
// wavefront and goes straight into MFMA operand registers - the dequantized weight never
// exists in memory.  Only the activations are shared.
//
// All global traffic of the main loop is asynchronous DMA into LDS (global_load_lds,
// 16 bytes per lane, no register staging), into a ring of D stages per workgroup:
//   - the BM x 64 slice of X for a k tile (read by every wavefront as MFMA operands).
//     Rows are not padded; the 16-byte chunk c of row r is stored at chunk position
//     c ^ (r & 7), which keeps the DMA writes and the 128-bit operand reads free of bank
//     conflicts;
//   - each wavefront's own 3 KB of packed planes per block of output channels
//     (lane-linear, exactly the order the planes have in memory).
// The DMA is issued from inline assembly and waited for with explicit s_waitcnt vmcnt:
// every step issues the same number of loads per wavefront, so "at most (D-2) groups
// still in flight" is a constant, and the compiler (which cannot see these loads) has
// no reason to drain the queue.  One barrier per k tile publishes the landed stage and
// frees the stage consumed in the previous step.
//
// LDS traffic per k tile: every wavefront reads the whole X slice (wavefronts x BM x 128 B) plus its
// planes - at BM = 128 about 152 KB per 2048 MFMA cycles of a SIMD, some 60 % of the 128 B/clk port.
// Measured, the loop keeps the matrix pipe busy 40-50 % of the time at BM = 128 and less at smaller BM,
// where a k tile holds too few MFMAs per barrier.  With the loads, the barrier, the unpack or the X
// reads taken out one at a time the loop gets no more than 10 % faster, and with all of them out 18 %:
// no single stage is the limit.  The shader clock under this kernel stays at 2.1-2.4 GHz of 2.4 on
// random data (zeros run up to 20 % faster on the shapes that fill all CUs, hardly at all on the
// others); where K is split, the meeting of the slices costs another 5-12 % at M = 512.
//
// The row scale is applied once, after the accumulation (Section 5.2).  K may be split
// over workgroups; the slices meet in an fp32 workspace exactly as in the decode kernel.
#pragma once

#include "fp6_common.hpp"
#include "fp6_internal.hpp"
#include "fp6_reduce.hpp"

#ifndef FP6_GEMM_HINTS
#define FP6_GEMM_HINTS 1
#endif

namespace fp6 {

constexpr int kWaveTileBytes = kHiTileBytes + kLoTileBytes;   // 3072: the planes of one 64x64 tile

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

// 4 bytes per lane from (base + lane_offset) to LDS address lds + 4 * lane.
__device__ __forceinline__ void dma4(const void* base, uint32_t lane_offset, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
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

// FGQ: one scale per `64 << gshift` elements along K (Section 3, fine-grained quantization).
// The product sums of the k tiles of one such block are formed in a second accumulator; at
// the end of the block they are multiplied by the block's scales and added to the running
// sum: the scale is applied to each block's finished product sum, and only then do the blocks
// accumulate (the fine-grained rule of Section 5.2).  The scales of
// a wavefront's 64 channels (128 bytes per block) ride along with every stage of the DMA ring.
// GBN = 64-wide blocks of output channels per workgroup: 8 (512 channels), or 4 for launches that would
// otherwise have too few workgroups.
// KW = K-ways inside the workgroup.  KW = 2 doubles the wavefronts: the second set (kh = 1) works on the same
// BM x (64 * GBN) block of Y one k tile further along, so a step covers two k tiles, and the two sets' sums are
// added in LDS after the main loop.  It is what two workgroups of a two-way K-split would do, with the meeting moved
// from the workspace into LDS: where K has to be split to fill the chip, half of the partial sums never leave the
// compute unit.  The ring then has DX stages for the activations (two k tiles each; they come from L2) and D stages
// for the planes (they come from HBM and need the longer lead).
template <int BM, int D, int WN, int DQ, bool FGQ, int FMT, int GBN, int KW = 1, int DX = D>
__global__ __launch_bounds__(GBN / WN * KW * 64, (GBN == 4 && KW == 1) ? 2 : 1) void gemm_kernel(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, int split_k, int gshift)
{
    static_assert(!FGQ || (WN == 1 && BM <= 64 && KW == 1), "fine-grained scales: two accumulators must fit the register file");
    static_assert(KW == 1 || (KW == 2 && WN == 1), "K-ways inside the workgroup: one or two");
    static_assert(DX >= 2 && DX <= D, "the activations never need a longer lead than the planes");
    constexpr int NWAVES = GBN / WN;                    // wavefronts side by side along N
    constexpr int WAVES = NWAVES * KW;
    constexpr int OUT_THREADS = NWAVES * 64;            // threads that hold the block of Y after the main loop
    constexpr int MT = BM / 16;                         // 16-row blocks of X per workgroup
    constexpr int NT = 4 * WN;                          // 16-channel blocks per wavefront
    constexpr int XG = KW * BM / 8;                     // 8-row groups (1 KB of DMA each) per stage: BM / 8 per k tile
    constexpr int XL = XG >= WAVES ? XG / WAVES : 1;    // X groups moved per wavefront and step
    constexpr int kLoads = XL + 3 * WN + (FGQ ? 1 : 0); // DMA instructions per wavefront and step
    constexpr int kXBytes = KW * BM * kTile * 2;
    constexpr int kPlaneBytes = GBN * KW * kWaveTileBytes + (FGQ ? WAVES * 256 : 0);   // per stage of the plane ring
    constexpr int kScaleOff = GBN * KW * kWaveTileBytes;          // FGQ: 256 bytes per wavefront, inside the plane stage
    constexpr int kPlaneBase = DX * kXBytes;                      // the plane ring follows the activation ring
    constexpr int kRingBytes = DX * kXBytes + D * kPlaneBytes;
    constexpr int kTileRegs = MT * NT * OUT_THREADS;    // float4 per output tile
    constexpr int kSumBytes = KW > 1 ? kTileRegs * 16 : 0;        // LDS for adding the two K-ways
    constexpr int kSmemBytes = kRingBytes > kSumBytes ? kRingBytes : kSumBytes;
    // loads that may still be in flight when a step starts: everything issued after the step's activations
    // (the rest of that step's loads and DX - 2 whole steps) and after its planes (D - 2 whole steps)
    constexpr int kInFlight = ((DX - 2) * kLoads + 3 * WN + (FGQ ? 1 : 0)) < ((D - 2) * kLoads)
                                  ? ((DX - 2) * kLoads + 3 * WN + (FGQ ? 1 : 0)) : ((D - 2) * kLoads);
    __shared__ __align__(16) unsigned char smem[kSmemBytes];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = KW > 1 ? wave / NWAVES : 0;          // which of the K-ways this wavefront works on
    const int nw = KW > 1 ? wave % NWAVES : wave;       // its position along N
    const int ktiles = K / kTile, nblocks = N / kTile;
    const int mblk = (M + BM - 1) / BM;
    const int nblk = (nblocks + GBN - 1) / GBN;
    // Workgroups are dealt round-robin to the eight compute dies, each with its own L2.  The
    // workgroups that read the same planes (same block of weights and K-slice, different rows of
    // X) get ids that are congruent mod 8, so they run on one die and the planes are fetched
    // into one L2 once.  It is the (weight block, K-slice) pairs that are dealt to the dies, so
    // that every die gets the same number of them, give or take one (dealing whole blocks left
    // two dies with twice the work at 10 blocks: 512 x 5120 x 13824 in three K-slices took 136 us, now 87).
    const int xcd = blockIdx.x & 7;
    int id = blockIdx.x >> 3;
    const int mb = id % mblk;
    id /= mblk;
    const int pair = id * 8 + xcd;
    if (pair >= nblk * split_k) return;      // the grid is padded to a multiple of eight pairs
    const int nbw = pair / split_k, s = pair % split_k;
    const int kt_per = ktiles / split_k;
    const int kt_begin = s * kt_per, kt_end = kt_begin + kt_per;
    const int m0 = mb * BM;
    const int nb0 = nbw * GBN + nw * WN;       // first block of output channels of this wavefront
    const int i = lane & 15, g = lane >> 4;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

    // X DMA: this wavefront moves the 8-row groups j = (wave*XL + p) % XG; group j belongs to k tile j / (BM/8)
    // of the step and holds rows 8 * (j % (BM/8)) .. +7; lane l of a group fetches row l/8 of them, chunk
    // (l%8) ^ (l/8), and lands at chunk position l%8.
    uint32_t xlane[XL], xlds[XL];
#pragma unroll
    for (int p = 0; p < XL; p++) {
        const int j = (wave * XL + p) % XG;
        int row = m0 + (j % (BM / 8)) * 8 + (lane >> 3);
        row = row < M ? row : M - 1;      // rows past M are computed on valid data and dropped
        xlane[p] = (uint32_t)row * (uint32_t)K * 2u + (uint32_t)(((lane & 7) ^ (lane >> 3)) * 16) +
                   (uint32_t)((j / (BM / 8)) * kTile * 2);
        xlds[p] = j * 1024;
    }
    const uint32_t wlane = lane * 16;
    const uint32_t wlds = wave * WN * kWaveTileBytes;       // inside a stage of the plane ring
    // blocks of channels past N are computed on the last valid block and dropped
    size_t tile0[WN];
#pragma unroll
    for (int c = 0; c < WN; c++) tile0[c] = (size_t)min(nb0 + c, nblocks - 1) * ktiles;

    // kLoads DMA instructions per call, always: the activations of the step that starts at k tile `ktx` into stage sx
    // of their ring, this wavefront's planes of the step that starts at `ktw` into stage sw of theirs
    auto issue = [&](int ktx, int sx, int ktw, int sw) {
        const uint32_t xs = smem_base + sx * kXBytes;
        const uint32_t sb = smem_base + kPlaneBase + sw * kPlaneBytes;
        const unsigned char* xb = reinterpret_cast<const unsigned char*>(X) + (size_t)ktx * (kTile * 2);
#pragma unroll
        for (int p = 0; p < XL; p++) dma16(xb, xlane[p], xs + xlds[p]);
        const int kt = ktw + kh;          // this wavefront's k tile of the step
#pragma unroll
        for (int c = 0; c < WN; c++) {
            const unsigned char* hb = reinterpret_cast<const unsigned char*>(hi) + (tile0[c] + kt) * kHiTileBytes;
            const unsigned char* lb = reinterpret_cast<const unsigned char*>(lo) + (tile0[c] + kt) * kLoBytesOf<FMT>;
            dma16(hb, wlane, sb + wlds + c * kWaveTileBytes);
            dma16(hb + 1024, wlane, sb + wlds + c * kWaveTileBytes + 1024);
            // FP5: the 1-bit plane has 512 bytes per tile; the upper lanes fetch them a second time
            // (into the unused half of the stage's 1 KB) rather than bytes of the next tile
            dma16(lb, FMT != kE3M1 ? wlane : (wlane & 511u), sb + wlds + c * kWaveTileBytes + 2048);
        }
        if (FGQ) {
            // scales of this tile's block for the wavefront's 64 channels: 128 bytes, fetched by lanes
            // 0..31 (the upper lanes fetch the same bytes again rather than bytes past the array)
            const unsigned char* sp = reinterpret_cast<const unsigned char*>(scales) +
                                      ((size_t)(kt >> gshift) * N + (size_t)min(nb0, nblocks - 1) * kTile) * 2;
            dma4(sp, (lane & 31) * 4, sb + kScaleOff + wave * 256);
        }
    };
    const int kt_last = kt_end - KW;      // first k tile of the last step (steps past it re-fetch it and are dropped)

    // operand reads: row r = 16a + i, chunk 4q + g, at position (4q + g) ^ (i & 7), in this wavefront's k tile of the stage
    const int xoff0 = kh * (BM * kTile * 2) + i * (kTile * 2) + ((g ^ (i & 7)) * 16);
    const int xoff1 = kh * (BM * kTile * 2) + i * (kTile * 2) + (((4 + g) ^ (i & 7)) * 16);

    float4v acc[MT][NT];
    float4v part[FGQ ? MT : 1][FGQ ? NT : 1];      // FGQ: product sums of the current block of K
#pragma unroll
    for (int a = 0; a < MT; a++)
#pragma unroll
        for (int t = 0; t < NT; t++) {
            acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
            if (FGQ) part[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
        }

    // prologue: the steps 0 .. D-2 of the planes; their activations only as far as the shorter ring reaches
    // (a call always issues kLoads loads: a slot that is not due yet fetches what step 0 needs once more)
#pragma unroll
    for (int u = 0; u < D - 1; u++) {
        const int ux = u < DX - 1 ? u : 0;
        issue(min(kt_begin + ux * KW, kt_last), ux, min(kt_begin + u * KW, kt_last), u);
    }

    // One step (KW k tiles).  Its planes were issued D-1 steps ago, its activations DX-1 steps ago; kInFlight younger
    // loads may stay in flight.  The stage numbers are compile-time constants (the loop below is unrolled over a
    // whole period of both rings), so every LDS address is a register plus an immediate - a ring indexed at run
    // time measured 10-20% slower.
    auto step = [&](int kt, int ux, int uw) {
        wait_vmcnt<kInFlight>();
        __syncthreads();          // everyone's DMA landed; everyone is done with the stages refilled next
        issue(min(kt + (DX - 1) * KW, kt_last), (ux + DX - 1) % DX, min(kt + (D - 1) * KW, kt_last), (uw + D - 1) % D);
        const unsigned char* st = smem + ux * kXBytes;
        const unsigned char* wt = smem + kPlaneBase + uw * kPlaneBytes + wlds;
        const unsigned char* sct = smem + kPlaneBase + uw * kPlaneBytes + kScaleOff;
        TileRaw raw[WN];
#pragma unroll
        for (int c = 0; c < WN; c++) {
            raw[c].hi0 = *reinterpret_cast<const u32x4*>(wt + c * kWaveTileBytes + wlane);
            raw[c].hi1 = *reinterpret_cast<const u32x4*>(wt + c * kWaveTileBytes + 1024 + wlane);
            if (FMT != kE3M1) {
                raw[c].lo = *reinterpret_cast<const u32x4*>(wt + c * kWaveTileBytes + 2048 + wlane);
            } else {
                const u32x2 l = *reinterpret_cast<const u32x2*>(wt + c * kWaveTileBytes + 2048 + lane * 8);
                raw[c].lo = u32x4{l.x, l.y, 0u, 0u};
            }
        }
#pragma unroll
        for (int q = 0; q < 2; q++) {
            half8 xf[MT];
#pragma unroll
            for (int a = 0; a < MT; a++) {
                xf[a] = *reinterpret_cast<const half8*>(st + a * 16 * (kTile * 2) + (q ? xoff1 : xoff0));
            }
#pragma unroll
            for (int c = 0; c < WN; c++) {
                half8 w4[4];
                if (layout2(FMT)) unpack_kblock<DQ, FMT>(raw[c], q, w4);     // all four fragments at once
#pragma unroll
                for (int t4 = 0; t4 < 4; t4++) {
                    const int t = 4 * c + t4;
                    half8 w = layout2(FMT) ? w4[t4] : unpack_tile_fragment<DQ, FMT>(raw[c], 2 * t4 + q);
#pragma unroll
                    for (int a = 0; a < MT; a++) {
                        if (FGQ) part[a][t] = mfma16x16x32_of<FMT>(w, xf[a], part[a][t]);
                        else acc[a][t] = mfma16x16x32_of<FMT>(w, xf[a], acc[a][t]);
                    }
                }
            }
        }
        if (FGQ) {
            // last tile of a block of K (or of this workgroup's K-slice): scale and accumulate
            if ((((kt + 1) >> gshift) << gshift) == kt + 1 || kt + 1 == kt_end) {
#pragma unroll
                for (int t = 0; t < NT; t++) {
                    const half4 h = *reinterpret_cast<const half4*>(sct + wave * 256 + (t * 16 + g * 4) * 2);
#pragma unroll
                    for (int a = 0; a < MT; a++) {
#pragma unroll
                        for (int r = 0; r < 4; r++) acc[a][t][r] += part[a][t][r] * (float)h[r];
                        part[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
        }
        // Issue order.  The wavefronts of a SIMD leave the barrier together, so they cannot hide
        // each other's unpack work; instead, after the first fragment, every MFMA (16 cycles in the
        // matrix pipe) is followed by two (BM = 128) or four of the unpack VALU operations (in its
        // shadow), and the LDS operand reads of the second k block are spread over the MFMAs of
        // the first.
#if FP6_GEMM_HINTS
        // (tuned for the instruction mix of the FP6 bias-shift unpack; the other variants are left to the compiler,
        // whose schedule needs fewer registers - and so are four-wavefront workgroups of 64 and 128 rows, whose two
        // wavefronts on a SIMD come from different workgroups and do not leave a barrier together: 2 % faster unhinted)
        if (!FGQ && FMT == kE3M2 && DQ != kHalfMul && (GBN * KW == 8 || BM == 32)) {
        __builtin_amdgcn_sched_group_barrier(0x100, 3 * WN + MT, 0);     // planes + operands of k block 0
        __builtin_amdgcn_sched_group_barrier(0x002, 15, 0);              // first fragment
#pragma unroll
        for (int n = 0; n < 2 * NT * MT; n++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, MT >= 8 ? 2 : 4, 0);     // measured: 4 is 2-3 % ahead at BM <= 64, 9 % behind at 128
            if (n % 2 == 0 && n >= NT * MT - 2 * MT && n < NT * MT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        }
#endif
    };

    constexpr int P = (D % DX == 0) ? D : D * DX;      // steps after which both rings are back at stage 0
    int kt = kt_begin;
    for (; kt + P * KW <= kt_end; kt += P * KW) {      // steady state: branch-free trips of P steps
#pragma unroll
        for (int u = 0; u < P; u++) step(kt + u * KW, u % DX, u % D);
    }
#pragma unroll
    for (int u = 0; u < P - 1; u++) {        // the remaining steps
        if (kt + u * KW < kt_end) step(kt + u * KW, u % DX, u % D);
    }
    wait_vmcnt<0>();     // the over-fetched ring slots must land before LDS is given back
    __syncthreads();

    // ---- the two K-ways of the workgroup: the second set of wavefronts hands its sums over in LDS and is done
    if (KW > 1) {
        float4v* sums = reinterpret_cast<float4v*>(smem);
        if (kh == 1) {
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < NT; t++) sums[(a * NT + t) * OUT_THREADS + nw * 64 + lane] = acc[a][t];
        }
        __syncthreads();
        if (kh == 0) {
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < NT; t++) acc[a][t] += sums[(a * NT + t) * OUT_THREADS + nw * 64 + lane];
        }
    }

    // Everything below is addressed through a copy of the thread index that the compiler cannot
    // see through, so that none of its address arithmetic is hoisted above the main loop, where it
    // would take registers the loop needs (and a spilled value reloaded inside the loop makes the
    // compiler drain the DMA queue).
    int tid2 = tid;
    asm volatile("" : "+v"(tid2));
    const int i2 = tid2 & 15, g2 = (tid2 >> 4) & 3;

    // ---- K-slices of other workgroups
    const bool holds_y = KW == 1 || kh == 0;       // (wave-uniform) the wavefronts that hold the block of Y
    if (split_k > 1) {
        const int tile = nbw * mblk + mb, ntiles = mblk * nblk;
        if (holds_y) {
            __amdgpu_buffer_rsrc_t win = partial_window(partials + ((size_t)s * ntiles + tile) * kTileRegs, kTileRegs * 16);
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < NT; t++) store_partial(win, (a * NT + t) * OUT_THREADS + tid2, acc[a][t]);
        }
        if (!arrive_last(&counters[tile * kCounterStride], (uint32_t)split_k)) return;
        if (!holds_y) return;
        // Two slices: the one that arrives last adds the other's sums to its own, which it still holds - a + b
        // does not depend on who that is.  More slices: all of them are read back and added in slice order.
        const bool two = split_k == 2;
        if (!two) {
#pragma unroll
            for (int a = 0; a < MT; a++)
#pragma unroll
                for (int t = 0; t < NT; t++) acc[a][t] = float4v{0.f, 0.f, 0.f, 0.f};
        }
        for (int ss = two ? 1 - s : 0; ss < (two ? 2 - s : split_k); ss++) {
            __amdgpu_buffer_rsrc_t win = partial_window(partials + ((size_t)ss * ntiles + tile) * kTileRegs, kTileRegs * 16);
            // sixteen 16-byte loads in flight at a time: more would need registers the main loop
            // cannot spare
            constexpr int AG = (MT * NT < 16) ? MT : 16 / NT;
#pragma unroll
            for (int a0 = 0; a0 < MT; a0 += AG) {
                float4v v[AG][NT];
#pragma unroll
                for (int a = 0; a < AG; a++)
#pragma unroll
                    for (int t = 0; t < NT; t++) v[a][t] = load_partial(win, ((a0 + a) * NT + t) * OUT_THREADS + tid2);
#pragma unroll
                for (int a = 0; a < AG; a++)
#pragma unroll
                    for (int t = 0; t < NT; t++) acc[a0 + a][t] += v[a][t];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else if (!holds_y) {
        return;
    }

    // ---- epilogue: lane holds channels n = 16t + 4g + r of row m = 16a + i  (i2, g2 = i, g)
#pragma unroll
    for (int c = 0; c < WN; c++) {
        const int nb = nb0 + c;
        if (nb >= nblocks) break;
        float sc[4][4];
#pragma unroll
        for (int t = 0; t < 4; t++) {
            half4 h = half4{1, 1, 1, 1};       // fine-grained scales were applied block by block
            if (!FGQ) h = *reinterpret_cast<const half4*>(scales + (size_t)nb * kTile + t * 16 + g2 * 4);
#pragma unroll
            for (int r = 0; r < 4; r++) sc[t][r] = (float)h[r] * kUnshift<DQ, FMT>;
        }
#pragma unroll
        for (int a = 0; a < MT; a++) {
            const int m = m0 + a * 16 + i2;
            if (m < M) {
#pragma unroll
                for (int t = 0; t < 4; t++) {
                    // (the fp16 branch is kept exactly as it was before bf16 came: routed through the same helper as the
                    // bf16 one, the 128-row eight-wavefront kernel spilled a second register, reloaded it inside the main
                    // loop, and the config-5 stack at M = 512 ran 5 % slower - 35.5 against 33.7 ms on one machine)
                    if constexpr (FMT == kE3M2B) {
                        float yv[4];
#pragma unroll
                        for (int r = 0; r < 4; r++) yv[r] = acc[a][c * 4 + t][r] * sc[t][r];
                        *reinterpret_cast<half4*>(Y + (size_t)m * N + (size_t)nb * kTile + t * 16 + g2 * 4) = to_out4<FMT>(yv);
                    } else {
                        half4 y;
#pragma unroll
                        for (int r = 0; r < 4; r++) y[r] = (_Float16)(acc[a][c * 4 + t][r] * sc[t][r]);
                        *reinterpret_cast<half4*>(Y + (size_t)m * N + (size_t)nb * kTile + t * 16 + g2 * 4) = y;
                    }
                }
            }
        }
    }
}

template <int BM, int D, int WN, int DQ = kBiasShift, bool FGQ = false, int FMT = kE3M2, int GBN = 8, int KW = 1, int DX = D>
static hipError_t launch_gemm_t(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                                const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                                hipStream_t stream)
{
    uint32_t* counters = reinterpret_cast<uint32_t*>(workspace);
    float4v* partials = reinterpret_cast<float4v*>(reinterpret_cast<char*>(workspace) + kZeroBytes);
    const int64_t mblk = (M + BM - 1) / BM, nblk = (N / kTile + GBN - 1) / GBN;
    const unsigned grid = (unsigned)(mblk * ((nblk * p.split_k + 7) / 8 * 8));   // padded: see the id mapping
    hipLaunchKernelGGL((gemm_kernel<BM, D, WN, DQ, FGQ, FMT, GBN, KW, DX>), dim3(grid), dim3(GBN / WN * KW * 64), 0, stream, X, (int)M,
                       (const u32x4*)hi, (const u32x4*)lo, scales, (int)N, (int)K, Y, partials, counters, p.split_k, p.gshift);
    return hipGetLastError();
}

}  // namespace fp6
