// Streaming (decode-shape) kernels of the W6A16 linear layer for gfx950: M <= 16, and up to 64 rows
// with several row blocks per wavefront.
//
// The work is a stream over the packed weight (0.75 byte per weight, Section 5.1):
// a workgroup owns 64 output channels and one K-slice; its wavefronts take the slice's
// 64x64 tiles round-robin, so the workgroup walks one contiguous region of each plane.
// Per tile a lane issues three 128-bit loads (two of the 4-bit plane, one of the 2-bit
// plane), pads the sub-numbers into fp16 operands in registers (bias shift, Section 5.2)
// and feeds eight v_mfma_f32_16x16x32_f16 (weights = A, the <=16 rows of X = B, padded
// with zero columns).  X is tiny and L2-resident, so each wavefront reads its 16-byte
// operand slices of X directly.  Partial sums of the wavefronts are added in LDS; if K
// is also split over workgroups the slices meet in the workspace - two slices pairwise in
// a slot, more at an arrival counter, where the workgroup that arrives last adds them in
// slice order (both deterministic) - and whoever holds the total applies the epilogue
// Y = fp16(acc * S_n * 2^12), the row scale after the accumulation (Section 5.2).
#include "fp6_common.hpp"
#include "fp6_internal.hpp"
#include "fp6_reduce.hpp"

namespace fp6 {

struct XFrag {
    half8 q0, q1;   // operand slices for the two 32-wide k blocks of a tile
};

// Lanes whose column m is past M read row M-1 instead: the MFMA columns are independent,
// so those columns only produce values that are never stored.
__device__ __forceinline__ XFrag load_x(const uint16_t* __restrict__ xrow, int kt)
{
    XFrag x;
    const half8* p = reinterpret_cast<const half8*>(xrow + (size_t)kt * kTile);
    x.q0 = p[0];
    x.q1 = p[4];   // +32 halfs
    return x;
}

// One tile against MB blocks of 16 rows of X: every fragment is unpacked once and used MB times.
template <int DQ, int FMT, int MB>
__device__ __forceinline__ void tile_mac(const TileRaw& r, const XFrag (&x)[MB], float4v (&acc)[MB][4])
{
    if (layout2(FMT)) {
        // layout 2: the unpack yields the four fragments of a k block at once
#pragma unroll
        for (int q = 0; q < 2; q++) {
            half8 w[4];
            unpack_kblock<DQ, FMT>(r, q, w);
#pragma unroll
            for (int t = 0; t < 4; t++)
#pragma unroll
                for (int c = 0; c < MB; c++) acc[c][t] = mfma16x16x32_of<FMT>(w[t], q ? x[c].q1 : x[c].q0, acc[c][t]);
        }
        return;
    }
#pragma unroll
    for (int f = 0; f < 8; f++) {
        half8 w = unpack_tile_fragment<DQ, FMT>(r, f);
#pragma unroll
        for (int c = 0; c < MB; c++) acc[c][f >> 1] = mfma16x16x32_of<FMT>(w, (f & 1) ? x[c].q1 : x[c].q0, acc[c][f >> 1]);
    }
}

// D = depth of the per-wavefront ring of tiles in flight (D-1 tiles are being fetched
// while one is consumed).  The ring is indexed with compile-time constants only.
// FGQ: one scale per `64 << gshift` elements along K (Section 3, fine-grained quantization)
// instead of one per row.  A tile lies inside one such block, so its product sums are
// formed in a zeroed accumulator and multiplied by the block's scales while they are added
// to the running sum: the scale meets the block's finished product sum before the blocks
// accumulate (the fine-grained rule of Section 5.2).
// The scales of the workgroup's 64 channels for its whole K-slice (128 bytes per block) are
// copied to LDS before the stream starts (one short wait at the head of the kernel).
// MB = blocks of 16 rows of X handled by every wavefront (M <= 16 * MB).  MB > 1 extends the stream to
// M <= 64: the weights are still read and unpacked once, X (L2-resident) is read MB times as much.
// nb = the workgroup's block of 64 output channels, s = its K-slice.  gnb = the index under which the block meets
// its other K-slices in the workspace: nb for a single layer; in a group of layers launched together, the block's
// index in the concatenation of their channel blocks.
template <int WAVES, int D, int DQ, bool FGQ, int FMT, int MB>
__device__ __forceinline__ void decode_block(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, unsigned long long* __restrict__ slots,
    int split_k, int pairwise, int gshift, int nb, int s, int gnb)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ktiles = K / kTile;
    const int kt_per = ktiles / split_k;
    const int kt_end = (s + 1) * kt_per;
    static_assert(MB == 1 || !FGQ, "several row blocks: row-wise scales only");
    const int m = lane & 15, g = lane >> 4;
    const uint16_t* xrow[MB];
#pragma unroll
    for (int c = 0; c < MB; c++) xrow[c] = X + (size_t)min(16 * c + m, M - 1) * K + g * 8;
    const size_t tile0 = (size_t)nb * ktiles;

    // row scales of the four channels this thread will store (fetched early: the epilogue is latency-bound)
    half4 sc = half4{1, 1, 1, 1};
    if (!FGQ && (int)threadIdx.x < 256) sc = *reinterpret_cast<const half4*>(scales + nb * kTile + (threadIdx.x & 15) * 4);

    float4v acc[MB][4];
#pragma unroll
    for (int c = 0; c < MB; c++)
#pragma unroll
        for (int t = 0; t < 4; t++) acc[c][t] = float4v{0.f, 0.f, 0.f, 0.f};

    // FGQ: this workgroup's scales -> LDS (16-byte pieces; piece c = block group0 + c/8, channels 8*(c%8)..+7),
    // four loads per thread in flight
    extern __shared__ __align__(16) uint16_t gscale[];
    const int group0 = (s * kt_per) >> gshift;
    if (FGQ) {
        constexpr int T = WAVES * 64;
        const int pieces = (((kt_end - 1) >> gshift) - group0 + 1) * 8;
        for (int c0 = threadIdx.x; c0 < pieces; c0 += 4 * T) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = min(c0 + u * T, pieces - 1);
                v[u] = *reinterpret_cast<const u32x4*>(scales + (size_t)(group0 + (c >> 3)) * N + nb * kTile + (c & 7) * 8);
            }
#pragma unroll
            for (int u = 0; u < 4; u++)
                if (c0 + u * T < pieces) *reinterpret_cast<u32x4*>(gscale + (c0 + u * T) * 8) = v[u];
        }
        __syncthreads();
    }

    // this wavefront's tiles: kt0, kt0 + WAVES, ...  (cnt of them, possibly none)
    const int kt0 = s * kt_per + wave;
    const int cnt = (kt_end - kt0 + WAVES - 1) / WAVES;
    if (cnt > 0) {
        TileRaw raw[D];
        XFrag xf[D][MB];
        auto fetch_x = [&](int slot, int k) {
#pragma unroll
            for (int c = 0; c < MB; c++) xf[slot][c] = load_x(xrow[c], k);
        };
        // k = the tile's index along K
        auto mac = [&](int slot, int k) {
            if (FGQ) {
                float4v part[MB][4];
#pragma unroll
                for (int t = 0; t < 4; t++) part[0][t] = float4v{0.f, 0.f, 0.f, 0.f};
                tile_mac<DQ, FMT, MB>(raw[slot], xf[slot], part);
                const uint16_t* sg = gscale + ((k >> gshift) - group0) * kTile + g * 4;
#pragma unroll
                for (int t = 0; t < 4; t++) {
                    const half4 sv = *reinterpret_cast<const half4*>(sg + 16 * t);
#pragma unroll
                    for (int r = 0; r < 4; r++) acc[0][t][r] += part[0][t][r] * (float)sv[r];
                }
            } else {
                tile_mac<DQ, FMT, MB>(raw[slot], xf[slot], acc);
            }
        };

        // prologue: tiles 0 .. D-2 (clamped: a short wavefront re-reads its last tile)
#pragma unroll
        for (int u = 0; u < D - 1; u++) {
            const int k = kt0 + min(u, cnt - 1) * WAVES;
            raw[u] = load_tile<FMT>(hi, lo, tile0 + k, lane);
            fetch_x(u, k);
        }
        // steady state, branch-free: D tiles per trip, each step refills the slot freed one step ago
        int j0 = 0;
        for (; j0 + 2 * D - 1 <= cnt; j0 += D) {
#pragma unroll
            for (int u = 0; u < D; u++) {
                const int k = kt0 + (j0 + u + D - 1) * WAVES;
                raw[(u + D - 1) % D] = load_tile<FMT>(hi, lo, tile0 + k, lane);
                fetch_x((u + D - 1) % D, k);
                mac(u, kt0 + (j0 + u) * WAVES);
            }
        }
        // drain: the remaining (< 2D-1) tiles, refilling only while tiles are left
#pragma unroll
        for (int v = 0; v < 2 * D - 2; v++) {
            const int j = j0 + v;
            if (j < cnt) {
                if (j + D - 1 < cnt) {
                    const int k = kt0 + (j + D - 1) * WAVES;
                    raw[(v + D - 1) % D] = load_tile<FMT>(hi, lo, tile0 + k, lane);
                    fetch_x((v + D - 1) % D, k);
                }
                mac(v % D, kt0 + j * WAVES);
            }
        }
    }

    // ---- add the wavefronts' partial sums in LDS
    // MFMA result layout: lane 16g + m of accumulator t holds channels 16t + 4g + r (r = 0..3)
    // of column m.  Thread m*16 + (4t + g) takes that value, so the threads of the valid
    // columns come first and a column's 64 channels sit in 16 consecutive threads.
    __shared__ float4v red[WAVES][256];
    const int tid = threadIdx.x;
    const int mm = tid >> 4, n4 = tid & 15;
    float4v sum[MB];
    bool active[MB];
#pragma unroll
    for (int c = 0; c < MB; c++) {
        if (c) __syncthreads();                      // everyone has read the previous block's sums
#pragma unroll
        for (int t = 0; t < 4; t++) red[wave][t * 64 + lane] = acc[c][t];
        __syncthreads();
        active[c] = tid < 16 * (M - 16 * c);         // rows 16c .. of X that exist (tid < 256 follows)
        if (MB > 1) active[c] = active[c] && tid < 256;
        sum[c] = float4v{0.f, 0.f, 0.f, 0.f};
        if (active[c]) {
            const int src = (n4 >> 2) * 64 + (n4 & 3) * 16 + mm;
#pragma unroll
            for (int w = 0; w < WAVES; w++) sum[c] += red[w][src];
        }
    }

    // ---- add the K-slices of other workgroups
    bool keep_lo = active[0], keep_hi = active[0];     // pairwise meeting: which halves of `sum` this thread finishes
    if (split_k > 1 && pairwise && MB == 1) {
        // pairwise meeting, two values per slot: thread tid owns slots 2*tid and 2*tid + 1 of a node
        if (active[0]) {
            const size_t node = (size_t)32 * M;          // 64-bit slots per tree node
            unsigned long long* mine = slots + (size_t)gnb * split_k * node + tid * 2;
            Pair p0{sum[0][0], sum[0][1]}, p1{sum[0][2], sum[0][3]};
            keep_lo = meet_tree(mine, node, s, split_k, p0);
            keep_hi = meet_tree(mine + 1, node, s, split_k, p1);
            sum[0] = float4v{p0.a, p0.b, p1.a, p1.b};
        }
    } else if (split_k > 1) {
        // meeting at a counter: the last arrival adds all slices in slice order
        constexpr uint32_t kSliceBytes = 4096u * MB;
#pragma unroll
        for (int c = 0; c < MB; c++)
            if (active[c])
                store_partial(partial_window(partials + ((size_t)gnb * split_k + s) * (256 * MB), kSliceBytes), c * 256 + tid, sum[c]);
        if (!arrive_last(&counters[gnb * kCounterStride], (uint32_t)split_k)) return;
#pragma unroll
        for (int c = 0; c < MB; c++) {
            if (!active[c]) continue;
            sum[c] = float4v{0.f, 0.f, 0.f, 0.f};
            // up to sixteen slices in flight at a time
            constexpr int G = MB == 1 ? 16 : 8;
            for (int ss = 0; ss < split_k; ss += G) {
                float4v v[G];
#pragma unroll
                for (int u = 0; u < G; u++) {
                    const int sl = min(ss + u, split_k - 1);
                    v[u] = load_partial(partial_window(partials + ((size_t)gnb * split_k + sl) * (256 * MB), kSliceBytes), c * 256 + tid);
                }
#pragma unroll
                for (int u = 0; u < G; u++)
                    if (ss + u < split_k) sum[c] += v[u];
            }
        }
    }

    // ---- epilogue: 16 consecutive threads store the 64 channels of one row of Y
#pragma unroll
    for (int c = 0; c < MB; c++) {
        const bool lo_ok = c ? active[c] : keep_lo, hi_ok = c ? active[c] : keep_hi;
        if (!(lo_ok || hi_ok)) continue;
        float yv[4];
#pragma unroll
        for (int r = 0; r < 4; r++) yv[r] = sum[c][r] * ((float)sc[r] * kUnshift<DQ, FMT>);
        const half4 y = to_out4<FMT>(yv);
        uint16_t* dst = Y + (size_t)(16 * c + mm) * N + nb * kTile + n4 * 4;
        if (lo_ok && hi_ok) {
            *reinterpret_cast<half4*>(dst) = y;
        } else if (lo_ok) {
            *reinterpret_cast<half2v*>(dst) = half2v{y[0], y[1]};
        } else {
            *reinterpret_cast<half2v*>(dst + 2) = half2v{y[2], y[3]};
        }
    }
}

template <int WAVES, int D, int DQ, bool FGQ, int FMT, int MB>
__global__ __launch_bounds__(WAVES * 64) void decode_kernel(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, unsigned long long* __restrict__ slots,
    int split_k, int pairwise, int gshift)
{
    const int nb = blockIdx.x / split_k, s = blockIdx.x % split_k;
    decode_block<WAVES, D, DQ, FGQ, FMT, MB>(X, M, hi, lo, scales, N, K, Y, partials, counters, slots, split_k, pairwise,
                                             gshift, nb, s, nb);
}

// ---- several layers in one launch
// Layers that read activations of the same height M and are independent of one another (the q, k, v projections
// of an attention block; the gate and up projections of a feed-forward block) can share one launch: the
// workgroups of all of them start together, so the small layers ride in the shadow of the large one instead of
// paying a launch each.  The launch treats the layers' channel blocks as one list (layer 0's blocks, then layer
// 1's, ...) and gives every block the same plan; a workgroup finds its layer by comparing its position in that
// list with the layers' first positions.
constexpr int kGroupMax = FP6_GROUP_MAX;
struct DecodeLayer {
    const uint16_t* X;
    const u32x4* hi;
    const u32x4* lo;
    const uint16_t* scales;
    uint16_t* Y;
    int N;
};
struct DecodeGroup {
    DecodeLayer layer[kGroupMax];
    int first_block[kGroupMax];       // index of the layer's first channel block in the list; INT_MAX for unused entries
};

// The layer of channel block `gnb`; the selects run on scalar registers (gnb is uniform in the workgroup).
__device__ __forceinline__ DecodeLayer layer_of(const DecodeGroup& g, int gnb, int* first)
{
    DecodeLayer a = g.layer[0];
    *first = 0;
#pragma unroll
    for (int i = 1; i < kGroupMax; i++) {
        if (gnb >= g.first_block[i]) {
            a = g.layer[i];
            *first = g.first_block[i];
        }
    }
    return a;
}

template <int WAVES, int D>
__global__ __launch_bounds__(WAVES * 64) void decode_group_kernel(
    DecodeGroup g, int M, int K, float4v* __restrict__ partials, uint32_t* __restrict__ counters,
    unsigned long long* __restrict__ slots, int split_k, int pairwise)
{
    const int gnb = __builtin_amdgcn_readfirstlane(blockIdx.x / split_k), s = blockIdx.x % split_k;
    int first;
    const DecodeLayer a = layer_of(g, gnb, &first);
    decode_block<WAVES, D, kBiasShift, false, kE3M2, 1>(a.X, M, a.hi, a.lo, a.scales, a.N, K, a.Y, partials, counters,
                                                        slots, split_k, pairwise, -1, gnb - first, s, gnb);
}

// ---------------------------------------------------------------------------------------------
// Half-tile workgroups: a workgroup owns 32 output channels (the upper or lower half of the 64
// that a tile covers) and, wherever that yields enough workgroups, the whole of K - so the result
// needs no meeting with other workgroups.  Of each tile a lane fetches the 16 bytes of the 4-bit
// plane and the 8 bytes of the 2-bit plane that belong to its half (fragments 4h .. 4h+3).  The
// two halves of a block of channels run on the same compute die (ids 8 apart), so the 2-bit plane,
// whose 16-byte pieces hold both halves, is fetched from HBM once.
struct HalfRaw {
    u32x4 hi;
    u32x2 lo;
};

// FP5: the 1-bit plane has 8 bytes per lane and tile, one dword per half (fragments 4h .. 4h+3).
template <int FMT>
__device__ __forceinline__ HalfRaw load_half(const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
                                             size_t tile_index, int lane, int h)
{
    HalfRaw r;
    r.hi = __builtin_nontemporal_load(hi + tile_index * kHiTileVec + h * 64 + lane);
    if (FMT == kE3M1) {
        r.lo = u32x2{__builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(lo) + (tile_index * 64 + lane) * 2 + h), 0u};
    } else {
        r.lo = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(lo + tile_index * kLoTileVec + lane) + h);
    }
    return r;
}

// h = which half of the block's 64 channels; nb, s, gnb as in decode_block.
template <int WAVES, int D, int FMT = kE3M2>
__device__ __forceinline__ void decode_half_block(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, unsigned long long* __restrict__ slots,
    int split_k, int pairwise, int h, int nb, int s, int gnb)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ktiles = K / kTile;
    const int kt_per = ktiles / split_k;
    const int kt_end = (s + 1) * kt_per;
    const int m = lane & 15, g = lane >> 4;
    const uint16_t* xrow = X + (size_t)min(m, M - 1) * K + g * 8;
    const size_t tile0 = (size_t)nb * ktiles;
    const int ch0 = nb * kTile + h * 32;                   // first channel of this workgroup

    half4 sc = half4{0, 0, 0, 0};
    if ((int)threadIdx.x < 8 * M) sc = *reinterpret_cast<const half4*>(scales + ch0 + (threadIdx.x & 7) * 4);

    float4v acc[2];
    acc[0] = acc[1] = float4v{0.f, 0.f, 0.f, 0.f};
    auto mac = [&](const HalfRaw& r, const XFrag& x) {
#pragma unroll
        for (int f = 0; f < 4; f++) {
            half8 w = FMT == kE3M1 ? unpack_fragment_e3m1(r.hi[f], r.lo[0], f)
                                   : unpack_fragment<kBiasShift>(r.hi[f], r.lo[f >> 1] >> (4 * (f & 1)));
            acc[f >> 1] = mfma16x16x32(w, (f & 1) ? x.q1 : x.q0, acc[f >> 1]);
        }
    };

    const int kt0 = s * kt_per + wave;
    const int cnt = (kt_end - kt0 + WAVES - 1) / WAVES;
    if (cnt > 0) {
        HalfRaw raw[D];
        XFrag xf[D];
#pragma unroll
        for (int u = 0; u < D - 1; u++) {
            const int k = kt0 + min(u, cnt - 1) * WAVES;
            raw[u] = load_half<FMT>(hi, lo, tile0 + k, lane, h);
            xf[u] = load_x(xrow, k);
        }
        int j0 = 0;
        for (; j0 + 2 * D - 1 <= cnt; j0 += D) {
#pragma unroll
            for (int u = 0; u < D; u++) {
                const int k = kt0 + (j0 + u + D - 1) * WAVES;
                raw[(u + D - 1) % D] = load_half<FMT>(hi, lo, tile0 + k, lane, h);
                xf[(u + D - 1) % D] = load_x(xrow, k);
                mac(raw[u], xf[u]);
            }
        }
#pragma unroll
        for (int v = 0; v < 2 * D - 2; v++) {
            const int j = j0 + v;
            if (j < cnt) {
                if (j + D - 1 < cnt) {
                    const int k = kt0 + (j + D - 1) * WAVES;
                    raw[(v + D - 1) % D] = load_half<FMT>(hi, lo, tile0 + k, lane, h);
                    xf[(v + D - 1) % D] = load_x(xrow, k);
                }
                mac(raw[v % D], xf[v % D]);
            }
        }
    }

    // thread m*8 + (4t + g) takes channels 16t + 4g + r of column m  (t = 0, 1)
    __shared__ float4v red[WAVES][128];
    red[wave][lane] = acc[0];
    red[wave][64 + lane] = acc[1];
    __syncthreads();
    const int tid = threadIdx.x;
    const bool active = tid < 8 * M;
    const int mm = tid >> 3, n4 = tid & 7;
    float4v sum = float4v{0.f, 0.f, 0.f, 0.f};
    if (active) {
        const int src = (n4 >> 2) * 64 + (n4 & 3) * 16 + mm;
#pragma unroll
        for (int w = 0; w < WAVES; w++) sum += red[w][src];
    }
    bool keep_lo = active, keep_hi = active;
    if (split_k > 1 && pairwise) {
        if (active) {
            const size_t node = (size_t)32 * M;          // the two halves share their block's tree nodes
            unsigned long long* mine = slots + (size_t)gnb * split_k * node + (h * 8 * M + tid) * 2;
            Pair p0{sum[0], sum[1]}, p1{sum[2], sum[3]};
            keep_lo = meet_tree(mine, node, s, split_k, p0);
            keep_hi = meet_tree(mine + 1, node, s, split_k, p1);
            sum = float4v{p0.a, p0.b, p1.a, p1.b};
        }
    } else if (split_k > 1) {
        if (active)
            store_partial(partial_window(partials + ((size_t)gnb * split_k + s) * 256, 4096), h * 128 + tid, sum);
        if (!arrive_last(&counters[(gnb * 2 + h) * kCounterStride], (uint32_t)split_k)) return;
        if (active) {
            sum = float4v{0.f, 0.f, 0.f, 0.f};
            for (int ss = 0; ss < split_k; ss += 16) {
                float4v v[16];
#pragma unroll
                for (int u = 0; u < 16; u++) {
                    const int sl = min(ss + u, split_k - 1);
                    v[u] = load_partial(partial_window(partials + ((size_t)gnb * split_k + sl) * 256, 4096), h * 128 + tid);
                }
#pragma unroll
                for (int u = 0; u < 16; u++)
                    if (ss + u < split_k) sum += v[u];
            }
        }
    }
    if (keep_lo || keep_hi) {
        half4 y;
#pragma unroll
        for (int r = 0; r < 4; r++) y[r] = (_Float16)(sum[r] * ((float)sc[r] * 4096.0f));
        uint16_t* dst = Y + (size_t)mm * N + ch0 + n4 * 4;
        if (keep_lo && keep_hi) {
            *reinterpret_cast<half4*>(dst) = y;
        } else if (keep_lo) {
            *reinterpret_cast<half2v*>(dst) = half2v{y[0], y[1]};
        } else {
            *reinterpret_cast<half2v*>(dst + 2) = half2v{y[2], y[3]};
        }
    }
}

template <int WAVES, int D, int FMT = kE3M2>
__global__ __launch_bounds__(WAVES * 64) void decode_half_kernel(
    const uint16_t* __restrict__ X, int M, const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
    const uint16_t* __restrict__ scales, int N, int K, uint16_t* __restrict__ Y,
    float4v* __restrict__ partials, uint32_t* __restrict__ counters, unsigned long long* __restrict__ slots,
    int split_k, int pairwise)
{
    // ids b and b + 8 are the two halves of one (block, slice) unit
    const int h = (blockIdx.x >> 3) & 1;
    const int unit = (blockIdx.x & 7) + 8 * (blockIdx.x >> 4);
    if (unit >= (N / kTile) * split_k) return;            // the grid is padded to a multiple of 16
    const int nb = unit / split_k, s = unit % split_k;
    decode_half_block<WAVES, D, FMT>(X, M, hi, lo, scales, N, K, Y, partials, counters, slots, split_k, pairwise, h, nb, s, nb);
}

// several layers in one launch (see decode_group_kernel); `units` = channel blocks of all layers x split_k
template <int WAVES, int D>
__global__ __launch_bounds__(WAVES * 64) void decode_half_group_kernel(
    DecodeGroup g, int M, int K, int units, float4v* __restrict__ partials, uint32_t* __restrict__ counters,
    unsigned long long* __restrict__ slots, int split_k, int pairwise)
{
    const int h = (blockIdx.x >> 3) & 1;
    const int unit = (blockIdx.x & 7) + 8 * (blockIdx.x >> 4);
    if (unit >= units) return;
    const int gnb = __builtin_amdgcn_readfirstlane(unit / split_k), s = unit % split_k;
    int first;
    const DecodeLayer a = layer_of(g, gnb, &first);
    decode_half_block<WAVES, D, kE3M2>(a.X, M, a.hi, a.lo, a.scales, a.N, K, a.Y, partials, counters, slots, split_k,
                                       pairwise, h, gnb - first, s, gnb);
}

template <int WAVES, int D, int FMT = kE3M2>
static hipError_t launch_decode_half_t(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                                       hipStream_t stream)
{
    uint32_t* counters = reinterpret_cast<uint32_t*>(workspace);
    float4v* partials = reinterpret_cast<float4v*>(reinterpret_cast<char*>(workspace) + kZeroBytes);
    unsigned long long* slots = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(workspace) + kCounterBytes);
    const int64_t units = (N / kTile) * p.split_k;
    const unsigned grid = (unsigned)((units + 7) / 8 * 16);
    hipLaunchKernelGGL((decode_half_kernel<WAVES, D, FMT>), dim3(grid), dim3(WAVES * 64), 0, stream, X, (int)M,
                       (const u32x4*)hi, (const u32x4*)lo, scales, (int)N, (int)K, Y, partials, counters, slots,
                       p.split_k, p.pairwise);
    return hipGetLastError();
}

template <int WAVES, int D, int DQ = kBiasShift, bool FGQ = false, int FMT = kE3M2, int MB = 1>
static hipError_t launch_decode_t(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                                  const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                                  hipStream_t stream)
{
    uint32_t* counters = reinterpret_cast<uint32_t*>(workspace);
    float4v* partials = reinterpret_cast<float4v*>(reinterpret_cast<char*>(workspace) + kZeroBytes);
    unsigned long long* slots = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(workspace) + kCounterBytes);
    const unsigned grid = (unsigned)((N / kTile) * p.split_k);
    // FGQ: 128 bytes of scales per block of K in a workgroup's slice (a slice may start inside a block)
    const size_t lds = FGQ ? (size_t)(((K / kTile / p.split_k - 1) >> p.gshift) + 2) * 128 : 0;
    hipLaunchKernelGGL((decode_kernel<WAVES, D, DQ, FGQ, FMT, MB>), dim3(grid), dim3(WAVES * 64), lds, stream, X, (int)M,
                       (const u32x4*)hi, (const u32x4*)lo, scales, (int)N, (int)K, Y, partials, counters, slots,
                       p.split_k, p.pairwise, p.gshift);
    return hipGetLastError();
}

hipError_t launch_decode(const LinearPlan& p, const uint16_t* X, int64_t M, const void* hi, const void* lo,
                         const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                         hipStream_t stream)
{
    if (p.block_m == 32) return launch_decode_t<4, 4, kBiasShift, false, kE3M2, 2>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.block_m == 64) return launch_decode_t<4, 3, kBiasShift, false, kE3M2, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.half_tiles && p.format == kE3M1) return launch_decode_half_t<4, 4, kE3M1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.half_tiles) {
        if (p.depth == 8) return launch_decode_half_t<4, 8>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        if (p.depth == 6) return launch_decode_half_t<4, 6>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        return launch_decode_half_t<4, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
    if (p.format == kE3M2H) return launch_decode_t<4, 4, kBiasShift, false, kE3M2H>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.format == kE3M2B) return launch_decode_t<4, 4, kBiasShift, false, kE3M2B>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.format == kE3M1) return launch_decode_t<4, 4, kBiasShift, false, kE3M1>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.gshift >= 0) return launch_decode_t<4, 4, kBiasShift, true>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.dequant == kIntRebias) return launch_decode_t<4, 4, kIntRebias>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    if (p.dequant == kHalfMul) return launch_decode_t<4, 4, kHalfMul>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    switch (p.waves * 10 + p.depth) {
        case 42: return launch_decode_t<4, 2>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 43: return launch_decode_t<4, 3>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 82: return launch_decode_t<8, 2>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 83: return launch_decode_t<8, 3>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        case 84: return launch_decode_t<8, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
        default: return launch_decode_t<4, 4>(p, X, M, hi, lo, scales, N, K, Y, workspace, stream);
    }
}

// One launch for `count` layers that share M and K (the plan `p` was made for their channel blocks taken together).
hipError_t launch_decode_group(const LinearPlan& p, int count, const GroupLayer* layers, int64_t M, int64_t K, void* workspace,
                               hipStream_t stream)
{
    uint32_t* counters = reinterpret_cast<uint32_t*>(workspace);
    float4v* partials = reinterpret_cast<float4v*>(reinterpret_cast<char*>(workspace) + kZeroBytes);
    unsigned long long* slots = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(workspace) + kCounterBytes);
    DecodeGroup g;
    int64_t blocks = 0;
    for (int i = 0; i < kGroupMax; i++) {
        const GroupLayer& l = layers[i < count ? i : 0];
        g.layer[i] = DecodeLayer{l.X, (const u32x4*)l.hi, (const u32x4*)l.lo, l.scales, l.Y, (int)l.N};
        g.first_block[i] = i < count ? (int)blocks : 0x7FFFFFFF;
        if (i < count) blocks += l.N / kTile;
    }
    const int64_t units = blocks * p.split_k;
    if (p.half_tiles) {
        const unsigned grid = (unsigned)((units + 7) / 8 * 16);
        hipLaunchKernelGGL((decode_half_group_kernel<4, 4>), dim3(grid), dim3(256), 0, stream, g, (int)M, (int)K, (int)units,
                           partials, counters, slots, p.split_k, p.pairwise);
    } else {
        hipLaunchKernelGGL((decode_group_kernel<4, 4>), dim3((unsigned)units), dim3(256), 0, stream, g, (int)M, (int)K,
                           partials, counters, slots, p.split_k, p.pairwise);
    }
    return hipGetLastError();
}

}  // namespace fp6
