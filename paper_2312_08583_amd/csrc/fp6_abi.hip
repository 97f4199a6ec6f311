// C ABI of the library (include/fp6_linear.h): argument checks, launch planning and
// dispatch.  Everything here runs on the host; no allocation, no synchronisation.
#include "../../include/fp6_linear.h"

#include "fp6_internal.hpp"

#include <cmath>
#include <mutex>

namespace fp6 {

// The runtime keeps the last error of any earlier call on this thread until somebody reads it; the launchers
// report hipGetLastError() after their launch, so it is read (and dropped) once before, or a failure of an
// unrelated earlier call would be reported as this call's.
static void forget_earlier_errors() { (void)hipGetLastError(); }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static bool shape_ok(int64_t N, int64_t K)
{
    return N > 0 && K > 0 && N % FP6_TILE == 0 && K % FP6_TILE == 0 && N <= (int64_t)1 << 30 &&
           K <= (int64_t)1 << 30 && N * K <= (int64_t)1 << 40;
}

// ---- the planner's fitted constants, all in one place
//
// Times are microseconds, rates bytes per microsecond.  Every figure was fitted on one MI355X to a sweep of forced
// plans (fp6_linear with FP6_HINT_* and a forced split_k, timed as replays of a captured graph); the sweep behind
// each group is named with it.  tests/test_plan_pins.py pins what the planner chooses with them.
struct PlanModel {
    // -- streaming kernel, fewer than 256 channel blocks.  M <= 16: 17 shapes from 1024 x 1024 to 8192 x 28672 at
    //    M = 1, every divisor of the k tiles up to 32, full and half tiles.  M = 24 ... 64: 21 shapes, same splits.
    double launch;              // fixed cost of a launch
    double stream16, stream64;  // what all workgroups together pull from HBM (up to 16 rows; two or four row blocks)
    double wg_full, wg_half, wg_half_fp5;   // what one workgroup pulls: 64 channels; 32 channels; 32 channels of FP5
    double wg_rows_exponent;    // more than 16 rows: a workgroup pulls wg_full x (16 / M)^this
    double meet_pair;           // two slices meeting pairwise
    double meet_base16, meet_slice16;       // counter meeting, up to 16 rows: base + per slice
    double meet_base64, meet_slice64;       // more rows: (base + per slice) x M / 16
    // -- streaming against tiled kernel (plain FP6): sizes measured at M = 32 and 64 on 4096 x 4096, 4096 x 11008,
    //    5120 x 5120, 28672 x 8192
    int64_t stream_to_32_weights;           // up to 32 rows the streaming kernel wins up to this many weights
    int64_t stream_to_64_blocks, stream_to_64_weights;   // up to 64 rows: up to this many channel blocks and weights
    // -- tiled kernel: every (rows per workgroup, width, split) on 12 shapes from 4096 x 4096 to 8192 x 28672 at
    //    M = 32 ... 512; the model's choice is 1 % behind the sweep's best on average, 7 % at worst
    double step[3];             // one k tile of an eight-wavefront workgroup with 32, 64, 128 rows
    double narrow_step;         // a four-wavefront workgroup takes this fraction of it ...
    double shared_unit;         // ... times this when two of them share a compute unit
    double slice[3];            // adding up one more slice's partial sums, per 32 / 64 / 128 rows (eight wavefronts)
    double round_fixed;         // set-up and epilogue of a workgroup
    double split_fixed;         // storing partial sums and the counter round trip, once the layer is split
    double hbm_tiled;           // HBM stream under the tiled kernel's access pattern
};
static constexpr PlanModel kModel = {
    2.5, 6.2e6, 3.87e6, 35e3, 29e3, 22e3, 0.565, 1.3, 1.4, 0.03, 0.5, 0.093,
    (int64_t)72 << 20, 64, (int64_t)1 << 27,
    {0.77, 0.993, 1.417}, 0.57, 1.964, {0.528, 1.588, 4.681}, 2.774, 3.216, 4.529e6,
};

// Number of K-slices for the decode family where the cost model below does not apply: layers of 256 channel
// blocks or more at up to 16 rows of X (measured on MI355X at M = 1: no split from 384 blocks on; below, two
// slices, which meet pairwise - cheaper than any larger number), eight-wavefront workgroups, very short K.
// Every wavefront keeps >= 2 tiles.
static int pick_decode_split(int64_t units, int64_t ktiles, int waves)
{
    if (units >= 384) return 1;
    if (units * 2 >= 256 && ktiles % 2 == 0 && ktiles / 2 >= 2 * waves) return 2;
    int best = 1;
    for (int64_t d = 1; d <= ktiles; d++) {
        if (ktiles % d) continue;
        if (ktiles / d < 2 * waves) break;
        best = (int)d;
        if (units * d >= 256) break;
    }
    return best;
}

// Layers with fewer than 256 channel blocks at up to 16 rows of X: the number of K-slices and the kind of
// workgroup (64 or 32 channels) that a small cost model likes best, in microseconds, constants fitted to
// measurements on MI355X at M = 1 (17 shapes from 1024 x 1024 to 8192 x 28672, every divisor of the k tiles up to
// 32): a launch costs 2.5 us; the planes stream at 6.2 TB/s, but one workgroup of four wavefronts at no more than
// 35 GB/s (29 GB/s with 32 channels), and a compute unit works through ceil(workgroups / 256) of them; two slices
// meet for 1.3 us, more for 1.4 + 0.03 per slice.  Against always asking for 256 workgroups this takes 11008 x 4096
// from 10.7 to 8.0 us, 5120 x 5120 from 9.2 to 6.8, 13824 x 5120 from 14.2 to 11.3, 5120 x 13824 from 15.9 to 12.8.
//
// With two or four 16-row blocks of X per wavefront (M > 16; 21 shapes at M = 24, 32, 48, 64) a workgroup is slower,
// 35 GB/s x (16 / M)^0.57, the stream reaches 3.9 TB/s, and the meeting moves M / 16 times the bytes:
// (0.5 + 0.09 per slice) x M / 16.  Mean distance from the best split of the sweep 1.5 % (the previous rule: 7 %).
static void plan_small_decode(int64_t M, int64_t nblocks, int64_t ktiles, int tile_bytes, int waves, int forced_split,
                              bool may_half, bool must_half, int* split_out, bool* half_out)
{
    double best = 1e30;
    *split_out = forced_split ? forced_split : 1;
    *half_out = must_half;
    const double bytes = (double)nblocks * (double)ktiles * tile_bytes;
    for (int half = must_half ? 1 : 0; half <= (may_half || must_half ? 1 : 0); half++) {
        for (int64_t d = forced_split ? forced_split : 1; d <= (forced_split ? forced_split : 32) && d <= ktiles; d++) {
            if (ktiles % d) continue;
            if (d > 1 && ktiles / d < 2 * waves) break;       // every wavefront keeps at least two tiles
            const int64_t wgs = nblocks * d * (half ? 2 : 1);
            const double rounds = (double)((wgs + 255) / 256);
            const bool rows16 = M <= 16;
            const PlanModel& c = kModel;
            const double stream = bytes / (rows16 ? c.stream16 : c.stream64);
            // (FP5 half tiles fetch the 1-bit plane four bytes a lane: their lower rate separates 8192 x 8192, where they win, from 8192 x 22016, where they lose)
            const double rate = rows16 ? (half ? (tile_bytes == 3072 ? c.wg_half : c.wg_half_fp5) : c.wg_full)
                                       : c.wg_full * pow(16.0 / (double)M, c.wg_rows_exponent);
            const double unit = rounds * (bytes / (double)wgs) / rate;
            const double meet = d == 1 ? 0.0
                                : rows16 ? (d == 2 ? c.meet_pair : c.meet_base16 + c.meet_slice16 * (double)d)
                                         : (c.meet_base64 + c.meet_slice64 * (double)d) * (double)M / 16.0;
            const double cost = c.launch + (stream > unit ? stream : unit) + meet;
            if (cost < best - 1e-9) {
                best = cost;
                *split_out = (int)d;
                *half_out = half != 0;
            }
        }
    }
}

// fine-grained blocks: 64 * 2^j elements, dividing K
static bool block_ok(int64_t K, int64_t block)
{
    return block >= FP6_TILE && block % FP6_TILE == 0 && ((block / FP6_TILE) & (block / FP6_TILE - 1)) == 0 && K % block == 0;
}

bool make_plan(int format, int64_t M, int64_t N, int64_t K, int64_t block, int variant, int split_k, LinearPlan* plan)
{
    const int64_t ktiles = K / FP6_TILE, nblocks = N / FP6_TILE;
    // tuning hints ride in the upper bits of `variant`; 0 = automatic
    const int hint_waves = (variant >> 8) & 0xF, hint_depth = (variant >> 12) & 0xF, hint_bm = ((variant >> 16) & 0xF) * 16,
              hint_meet = (variant >> 20) & 0x3, hint_dequant = (variant >> 22) & 0x3,
              hint_half = (variant >> 24) & 0x3, hint_gbn = (variant >> 26) & 0xF, hint_kw = (variant >> 30) & 0x1;
    const int variant_hints = variant >> 8;
    variant &= 0xFF;
    if (variant == FP6_VARIANT_AUTO) {
        // The streaming kernel reads X once per wavefront and tile: unbeatable up to 16 rows, still ahead of the
        // tiled kernel up to 32 rows on layers of up to 72 M weights (4096 x 4096: 9.6 against 12.8 us), behind it
        // on larger ones (28672 x 8192: 48 against 40 us), where the tiled kernel's shared X tile pays.
        // Up to 64 rows it stays ahead where there are at most 64 channel blocks, too few tiles for the tiled kernel
        // (M = 64: 15.4 against 16.2 us at 4096 x 4096, 23.3 against 27.0 at 4096 x 11008; behind from 5120 channels on).
        const bool plain_call = format == kE3M2 && !block && !(variant_hints);
        const bool stream = M <= 16 || (M <= 32 && plain_call && N * K <= kModel.stream_to_32_weights) ||
                            (M <= 64 && plain_call && nblocks <= kModel.stream_to_64_blocks && N * K <= kModel.stream_to_64_weights);
        variant = stream ? FP6_VARIANT_DECODE : FP6_VARIANT_GEMM;
    }
    if (variant != FP6_VARIANT_DECODE && variant != FP6_VARIANT_GEMM) return false;
    if (variant == FP6_VARIANT_DECODE && M > 64) return false;
    if (split_k < 0 || (split_k > 0 && ktiles % split_k != 0)) return false;

    LinearPlan p{};
    p.kw = 1;
    p.variant = variant;
    p.dequant = hint_dequant;
    p.format = format;
    // the five-bit format exists for the default kernel configurations, row-wise scales only
    if (format != kE3M2 && (block || hint_dequant || hint_waves || hint_depth)) return false;
    p.gshift = -1;
    if (block) {
        if (!block_ok(K, block) || hint_dequant || hint_waves || hint_depth) return false;
        for (int64_t b = block / FP6_TILE; b; b >>= 1) p.gshift++;
    }
    // the ablations exist for the default kernel configurations only
    if (hint_dequant > 2 || (hint_dequant && (hint_waves || hint_depth))) return false;
    if (hint_half && variant != FP6_VARIANT_DECODE) return false;
    if (hint_kw && variant != FP6_VARIANT_GEMM) return false;
    if (hint_gbn && (variant != FP6_VARIANT_GEMM || hint_dequant || hint_waves || (hint_gbn != 8 && hint_gbn != 4)))
        return false;
    // 64-channel blocks (= wavefronts) per workgroup of the tiled kernel.  Eight share the activations best;
    // four give twice the workgroups where there are few (measured: 40 against 47 us at 32 x 28672 x 8192, 24
    // against 30 us at 512 x 1024 x 8192, 20.7 against 30 us at 128 x 5120 x 5120).  The cost model below chooses.
    const bool plain = format == kE3M2 && !block && !hint_dequant;
    const bool narrow_ok = !hint_dequant && variant == FP6_VARIANT_GEMM;      // every format but the ablations
    int64_t gbn = hint_gbn ? hint_gbn : 8;
    p.gbn = (int)gbn;
    int64_t tiles, regs_per_tile;
    if (variant == FP6_VARIANT_DECODE) {
        // half-tile workgroups (32 channels): plain FP6 with row scales and the bias-shift unpack only
        const bool half_ok = (format == kE3M2 || format == kE3M1) && !block && !hint_dequant &&
                             (!hint_waves || hint_waves == 4) && 2 * nblocks <= kMaxCounters;
        if (hint_half > 2 || (hint_half == 1 && !half_ok)) return false;
        // Measured at M <= 4: half-tile workgroups win where they give about one workgroup per compute unit with
        // no K-split or a two-way one (10.3 against 11.6 us at 8192 x 8192); with more workgroups per unit they lose.
        int model_split = 0;
        bool model_half = false;
        const int waves_now = hint_waves ? hint_waves : 4;
        if ((M <= 16 ? nblocks < 256 : true) && !hint_depth && waves_now == 4 && ktiles >= 8) {
            const bool may_half = half_ok && M <= 4 && hint_half != 2;
            plan_small_decode(M, nblocks, ktiles, format == kE3M1 ? 2560 : 3072, waves_now, split_k, may_half,
                              hint_half == 1, &model_split, &model_half);
        }
        p.half_tiles = hint_half == 1 || (hint_half == 0 && model_half);
        if ((hint_waves && hint_waves != 4 && hint_waves != 8) || hint_bm || hint_meet > 2 ||
            (hint_depth && !(p.half_tiles ? (hint_depth == 4 || hint_depth == 6 || hint_depth == 8)
                                          : (hint_depth >= 2 && hint_depth <= 4))))
            return false;
        // M > 16: the wavefronts take two or four blocks of 16 rows of X (plain FP6, default configuration only)
        p.block_m = M <= 16 ? 16 : (M <= 32 ? 32 : 64);
        if (M > 16 && (!plain || hint_waves || hint_depth || p.half_tiles || hint_meet == 2)) return false;
        p.waves = hint_waves ? hint_waves : 4;
        p.depth = hint_depth ? hint_depth : (p.block_m == 64 ? 3 : 4);      // four row blocks per wavefront: ring of three
        tiles = nblocks;
        regs_per_tile = 16 * p.block_m;            // float4 per output tile (64 channels x block_m rows, fp32)
        p.split_k = split_k ? split_k
                    : model_split ? model_split
                    : pick_decode_split(p.half_tiles ? 2 * nblocks : nblocks, ktiles, p.waves);
        if (block) {
            // the scales of a workgroup's K-slice are staged in LDS, 128 bytes per block of K: keep that under 96 KB
            auto lds = [&](int64_t d) { return (((ktiles / d - 1) >> p.gshift) + 2) * 128; };
            if (lds(p.split_k) > 96 * 1024) {
                if (split_k) return false;
                int64_t d = p.split_k;
                while (d <= ktiles && (ktiles % d || lds(d) > 96 * 1024)) d++;
                if (d > ktiles) return false;
                p.split_k = (int)d;
            }
        }
    } else {
        if ((hint_waves && hint_waves != 8) || hint_depth || hint_meet ||
            (hint_bm && hint_bm != 32 && hint_bm != 64 && hint_bm != 128))
            return false;
        if (M * K * 2 >= ((int64_t)1 << 32)) return false;   // X is addressed with 32-bit lane offsets
        p.waves = hint_waves ? hint_waves : 8;
        // Pick rows per workgroup, workgroup width and the number of K-slices with a small cost model
        // (microseconds; constants fitted on MI355X to a sweep of every plan on 12 shapes from 4096 x 4096 to
        // 8192 x 28672 at M = 32 ... 512: the model's choice is 1 % behind the best plan on average, 7 % at
        // worst).  One eight-wavefront workgroup or two four-wavefront ones are resident per compute unit, and the
        // (weight block, K-slice) pairs are dealt to the eight dies of 32 units each, so the launch takes
        // ceil(pairs per die x row blocks / (32 or 64)) rounds;
        // a round costs its k tiles at the per-tile time of the workgroup shape (or of the HBM stream, whichever
        // is longer) plus a fixed part that grows with the number of slices the last workgroup of a tile adds up.
        double best_cost = 0.0;
        if (block && hint_bm > 64) return false;        // fine-grained scales: two accumulators per tile
        int64_t best_gbn = gbn;
        for (int64_t g = 8; g >= 4; g -= 4) {
            if (hint_gbn ? g != hint_gbn : (g == 4 && !narrow_ok)) continue;
            for (int bm = 32; bm <= (block ? 64 : 128); bm *= 2) {
                if (hint_bm ? bm != hint_bm : (bm > 32 && bm / 2 >= M)) continue;
                const int64_t mblk = (M + bm - 1) / bm, nblk = (nblocks + g - 1) / g, t = mblk * nblk;
                const PlanModel& c = kModel;
                const int bi = bm == 128 ? 2 : (bm == 64 ? 1 : 0);
                const double step1 = c.step[bi] * (g == 8 ? 1.0 : c.narrow_step);
                const double slice = c.slice[bi] * (double)g / 8.0;
                const int64_t cap = g == 4 ? 2 : 1;          // four-wavefront workgroups: two per compute unit
                for (int64_t d = 1; d <= ktiles && d <= 64; d++) {
                    if (ktiles % d || (split_k && d != split_k)) continue;
                    if (d > 1 && t > kMaxCounters) break;
                    const int64_t wgs = t * d, resident = wgs < 256 * cap ? wgs : 256 * cap;
                    const int64_t per_die = (nblk * d + 7) / 8 * mblk;
                    const int64_t rounds = (per_die + 32 * cap - 1) / (32 * cap);
                    const double step = step1 * (cap == 2 && per_die > 32 ? c.shared_unit : 1.0);   // two sharing a unit
                    const double hbm_step = 3072.0 * (double)g * (double)resident / (double)mblk / c.hbm_tiled;
                    const double cost = (double)rounds * ((double)(ktiles / d) * (step > hbm_step ? step : hbm_step) + c.round_fixed +
                                                          (d > 1 ? c.split_fixed + (double)d * slice : 0.0));
                    if (best_cost == 0.0 || cost < best_cost) {
                        best_cost = cost;
                        p.block_m = bm;
                        p.split_k = (int)d;
                        best_gbn = g;
                    }
                }
            }
        }
        if (best_cost == 0.0) return false;
        gbn = best_gbn;
        p.gbn = (int)gbn;
        if (hint_kw) {
            // two K-ways inside the workgroup: plain FP6, 128 x 256 blocks, an even number of k tiles per slice
            if (!plain || gbn != 4 || p.block_m != 128 || (ktiles / p.split_k) % 2) return false;
            p.kw = 2;
        } else if (plain && !variant_hints && !split_k && p.block_m == 128 && p.split_k > 1 &&
                   ((M + 127) / 128) * ((nblocks + 3) / 4) <= kMaxCounters) {
            // Where the model splits K, two of the K-ways can stay inside a workgroup of 128 x 256 (eight wavefronts
            // that add their sums in LDS): the same workgroups and the same work per compute unit, with half the partial
            // sums travelling through the workspace.  Measured at M = 512: 8192 x 22016 in four slices 170 -> 153 us,
            // 8192 x 8192 in two slices 70.6 -> 67.5 us; 22016 x 8192, which is not split, stays as it is.
            const int64_t mblk = (M + 127) / 128, wgs4 = mblk * ((nblocks + 3) / 4) * p.split_k;
            if (gbn == 8 && p.split_k % 2 == 0) {
                gbn = 4;
                p.split_k /= 2;
                p.kw = 2;
            } else if (gbn == 4 && wgs4 >= 512 && p.split_k % 2 == 0) {
                p.split_k /= 2;
                p.kw = 2;
            } else if (gbn == 4 && wgs4 <= 256 && (ktiles / p.split_k) % 2 == 0) {
                p.kw = 2;
            }
            p.gbn = (int)gbn;
        }
        p.depth = gbn == 8 || p.kw == 2 ? (p.block_m == 128 ? 3 : 4) : (p.block_m == 128 ? 2 : (p.block_m == 64 ? 3 : 4));
        p.waves = (int)gbn * p.kw;
        tiles = ((M + p.block_m - 1) / p.block_m) * ((nblocks + gbn - 1) / gbn);
        regs_per_tile = (int64_t)(p.block_m / 16) * 4 * 64 * gbn;
    }
    if (p.split_k > 1) {
        if (tiles > kMaxCounters) {
            if (split_k) return false;             // forced split that the counters cannot serve
            p.split_k = 1;
        }
    }
    // the launch grid is tiles * split_k workgroups (doubled for half tiles, padded to a multiple of 16)
    if (tiles * p.split_k > ((int64_t)1 << 29)) return false;
    if (p.split_k > 1) {
        // Decode: two slices meet pairwise (one memory round trip instead of three) if the tree nodes,
        // 256 * M bytes each, fit the slot region; deeper trees measured slower than the counter.
        const bool fits = M <= 16 && (int64_t)p.split_k * tiles * 256 * M <= (int64_t)kSlotBytes;
        if (variant == FP6_VARIANT_DECODE && hint_meet == 2 && !fits) return false;
        p.pairwise = variant == FP6_VARIANT_DECODE && fits && (hint_meet ? hint_meet == 2 : p.split_k == 2);
        if (!p.pairwise) {
            p.counters = (int)tiles;
            p.partial_bytes = (size_t)p.split_k * (size_t)tiles * (size_t)regs_per_tile * 16u;
        }
    }
    *plan = p;
    return true;
}

static size_t plan_workspace(const LinearPlan& p) { return p.split_k > 1 ? kZeroBytes + p.partial_bytes : 0; }

}  // namespace fp6

using namespace fp6;

// ---- the workspace of fp6_linear_static: device memory that belongs to the library
//
// Each GPU the library runs on holds its own copy of this array, at its own address, until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the device address is
// looked up once per device (with that device current) and kept in scratch_ptr[]; kernels, and the fill
// below, are given that address and never the name.
static __device__ __align__(256) unsigned char scratch[FP6_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static void* scratch_ptr[kMaxDevices];        // device address of `scratch` on device d (NULL: not looked up yet)
static std::mutex scratch_mutex;

// grid-stride fill with zeros, 16 bytes per thread and trip (a kernel, not a memset node: callers may be capturing)
static __global__ void zero_fill_kernel(uint4* __restrict__ p, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = uint4{0u, 0u, 0u, 0u};
}

// Device address of this device's scratch; on the first call per device also clears the counters and slots
// at its start (on `stream`, ahead of the caller's launch).  Returns NULL on a HIP error.
static void* static_scratch(hipStream_t stream)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        (void)hipGetLastError();
        hipLaunchKernelGGL(zero_fill_kernel, dim3(256), dim3(256), 0, stream, reinterpret_cast<uint4*>(ptr), kZeroBytes / 16);
        if (hipGetLastError() != hipSuccess) return nullptr;
        scratch_ptr[dev] = ptr;
    }
    return scratch_ptr[dev];
}

// block == 0: one scale per row
static int quantize_pack_any(int format, const uint16_t* W, int64_t N, int64_t K, int64_t block, void* hi_plane, void* lo_plane,
                             uint16_t* scales, void* stream)
{
    if (!W || !hi_plane || !lo_plane || !scales) return FP6_ERR_NULL;
    if (!shape_ok(N, K) || (block && !block_ok(K, block))) return FP6_ERR_SHAPE;
    if (block && N * (K / block) > ((int64_t)1 << 30)) return FP6_ERR_SHAPE;      // one workgroup per scale
    if (!aligned16(W) || !aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(scales)) return FP6_ERR_ALIGN;
    forget_earlier_errors();
    return launch_quantize_pack(format, W, N, K, block ? block : K, hi_plane, lo_plane, scales, (hipStream_t)stream) ==
                   hipSuccess
               ? FP6_OK
               : FP6_ERR_HIP;
}

static int dequantize_any(int format, const void* hi_plane, const void* lo_plane, const uint16_t* scales, int64_t N, int64_t K,
                          int64_t block, uint16_t* W_hat, void* stream)
{
    if (!hi_plane || !lo_plane || !scales || !W_hat) return FP6_ERR_NULL;
    if (!shape_ok(N, K) || (block && !block_ok(K, block))) return FP6_ERR_SHAPE;
    if (!aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(scales) || !aligned16(W_hat)) return FP6_ERR_ALIGN;
    forget_earlier_errors();
    return launch_dequantize(format, hi_plane, lo_plane, scales, N, K, block ? block : K, W_hat, (hipStream_t)stream) ==
                   hipSuccess
               ? FP6_OK
               : FP6_ERR_HIP;
}

static size_t workspace_any(int format, int64_t M, int64_t N, int64_t K, int64_t block, int variant, int split_k)
{
    LinearPlan p;
    if (M <= 0 || M > (int64_t)1 << 24 || !shape_ok(N, K) || !make_plan(format, M, N, K, block, variant, split_k, &p)) return 0;
    return plan_workspace(p);
}

static int linear_any(int format, const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane,
                      const uint16_t* scales, int64_t N, int64_t K, int64_t block, uint16_t* Y, void* workspace,
                      size_t workspace_bytes, void* stream, int variant, int split_k)
{
    if (!X || !hi_plane || !lo_plane || !scales || !Y) return FP6_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24 || !shape_ok(N, K) || block < 0) return FP6_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(scales) || !aligned16(Y) ||
        !aligned16(workspace))
        return FP6_ERR_ALIGN;
    LinearPlan p;
    if (!make_plan(format, M, N, K, block, variant, split_k, &p)) return FP6_ERR_VARIANT;
    const size_t need = plan_workspace(p);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FP6_ERR_WORKSPACE;
    forget_earlier_errors();
    hipError_t e = (p.variant == FP6_VARIANT_DECODE)
                       ? launch_decode(p, X, M, hi_plane, lo_plane, scales, N, K, Y, workspace, (hipStream_t)stream)
                       : launch_gemm(p, X, M, hi_plane, lo_plane, scales, N, K, Y, workspace, (hipStream_t)stream);
    return e == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

// A group of layers can share one launch if the streaming kernel serves them (M <= 16) and they have one K:
// their channel blocks are then planned as the blocks of one layer with the summed N.
static bool group_shares_a_launch(int64_t M, const fp6_linear_problem* pr, int count, LinearPlan* plan)
{
    if (count < 2 || M > 16) return false;
    int64_t n_total = 0;
    for (int i = 0; i < count; i++) {
        if (pr[i].K != pr[0].K) return false;
        n_total += pr[i].N;
    }
    if (!shape_ok(n_total, pr[0].K)) return false;
    if (!make_plan(kE3M2, M, n_total, pr[0].K, 0, FP6_VARIANT_AUTO, 0, plan)) return false;
    return plan->variant == FP6_VARIANT_DECODE && plan->block_m == 16 && plan->waves == 4 && plan->depth == 4;
}

static int group_check(int64_t M, const fp6_linear_problem* pr, int count)
{
    if (!pr) return FP6_ERR_NULL;
    if (count < 1 || count > FP6_GROUP_MAX || M <= 0 || M > (int64_t)1 << 24) return FP6_ERR_SHAPE;
    for (int i = 0; i < count; i++) {
        if (!pr[i].X || !pr[i].hi_plane || !pr[i].lo_plane || !pr[i].scales || !pr[i].Y) return FP6_ERR_NULL;
        if (!shape_ok(pr[i].N, pr[i].K)) return FP6_ERR_SHAPE;
        if (!aligned16(pr[i].X) || !aligned16(pr[i].hi_plane) || !aligned16(pr[i].lo_plane) || !aligned16(pr[i].scales) ||
            !aligned16(pr[i].Y))
            return FP6_ERR_ALIGN;
    }
    return FP6_OK;
}

extern "C" {

int fp6_layout_version(void) { return FP6_LAYOUT_VERSION; }

const char* fp6_status_string(int status)
{
    switch (status) {
        case FP6_OK: return "ok";
        case FP6_ERR_NULL: return "a required pointer is NULL";
        case FP6_ERR_SHAPE: return "M, N, K must be positive, N and K multiples of 64, a scale block 64 * 2^j dividing K";
        case FP6_ERR_ALIGN: return "buffer pointers must be 16-byte aligned";
        case FP6_ERR_WORKSPACE: return "workspace missing or too small";
        case FP6_ERR_VARIANT: return "kernel variant or split_k not valid for this shape";
        case FP6_ERR_HIP: return "HIP launch error";
        case FP6_ERR_SCRATCH: return "this shape needs more than the FP6_STATIC_SCRATCH_BYTES of built-in scratch: use fp6_linear with a workspace";
        default: return "unknown status";
    }
}

int fp6_packed_sizes(int64_t N, int64_t K, size_t* hi_bytes, size_t* lo_bytes, size_t* scale_bytes)
{
    if (!shape_ok(N, K)) return FP6_ERR_SHAPE;
    if (hi_bytes) *hi_bytes = (size_t)(N * K / 2);
    if (lo_bytes) *lo_bytes = (size_t)(N * K / 4);
    if (scale_bytes) *scale_bytes = (size_t)(2 * N);
    return FP6_OK;
}

int fp6_quantize_pack(const uint16_t* W, int64_t N, int64_t K, void* hi_plane, void* lo_plane, uint16_t* scales,
                      void* stream)
{
    return quantize_pack_any(kE3M2, W, N, K, 0, hi_plane, lo_plane, scales, stream);
}

int fp6_quantize_pack_fgq(const uint16_t* W, int64_t N, int64_t K, int64_t block, void* hi_plane, void* lo_plane,
                          uint16_t* scales, void* stream)
{
    if (block <= 0) return FP6_ERR_SHAPE;
    return quantize_pack_any(kE3M2, W, N, K, block, hi_plane, lo_plane, scales, stream);
}

int fp6_unpack_codes(const void* hi_plane, const void* lo_plane, int64_t N, int64_t K, uint8_t* codes, void* stream)
{
    if (!hi_plane || !lo_plane || !codes) return FP6_ERR_NULL;
    if (!shape_ok(N, K)) return FP6_ERR_SHAPE;
    if (!aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(codes)) return FP6_ERR_ALIGN;
    forget_earlier_errors();
    return launch_unpack_codes(kE3M2, hi_plane, lo_plane, N, K, codes, (hipStream_t)stream) == hipSuccess
               ? FP6_OK
               : FP6_ERR_HIP;
}

int fp6_dequantize(const void* hi_plane, const void* lo_plane, const uint16_t* scales, int64_t N, int64_t K,
                   uint16_t* W_hat, void* stream)
{
    return dequantize_any(kE3M2, hi_plane, lo_plane, scales, N, K, 0, W_hat, stream);
}

int fp6_dequantize_fgq(const void* hi_plane, const void* lo_plane, const uint16_t* scales, int64_t N, int64_t K,
                       int64_t block, uint16_t* W_hat, void* stream)
{
    if (block <= 0) return FP6_ERR_SHAPE;
    return dequantize_any(kE3M2, hi_plane, lo_plane, scales, N, K, block, W_hat, stream);
}

size_t fp6_linear_variant_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int split_k)
{
    return workspace_any(kE3M2, M, N, K, 0, variant, split_k);
}

size_t fp6_linear_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    return workspace_any(kE3M2, M, N, K, 0, FP6_VARIANT_AUTO, 0);
}

size_t fp6_linear_fgq_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t block, int variant, int split_k)
{
    return block > 0 ? workspace_any(kE3M2, M, N, K, block, variant, split_k) : 0;
}

size_t fp6_linear_group_workspace_bytes(int64_t M, const fp6_linear_problem* problems, int count)
{
    if (group_check(M, problems, count) != FP6_OK) return 0;
    LinearPlan p;
    if (group_shares_a_launch(M, problems, count, &p)) return plan_workspace(p);
    size_t need = 0;
    for (int i = 0; i < count; i++) {
        const size_t n = workspace_any(kE3M2, M, problems[i].N, problems[i].K, 0, FP6_VARIANT_AUTO, 0);
        need = n > need ? n : need;
    }
    return need;
}

int fp6_linear_group(int64_t M, const fp6_linear_problem* problems, int count, void* workspace, size_t workspace_bytes,
                     void* stream)
{
    const int bad = group_check(M, problems, count);
    if (bad != FP6_OK) return bad;
    if (!aligned16(workspace)) return FP6_ERR_ALIGN;
    const size_t need = fp6_linear_group_workspace_bytes(M, problems, count);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FP6_ERR_WORKSPACE;
    LinearPlan p;
    if (group_shares_a_launch(M, problems, count, &p)) {
        GroupLayer layers[FP6_GROUP_MAX];
        for (int i = 0; i < count; i++)
            layers[i] = GroupLayer{problems[i].X, problems[i].hi_plane, problems[i].lo_plane, problems[i].scales, problems[i].Y,
                                   problems[i].N};
        forget_earlier_errors();
        return launch_decode_group(p, count, layers, M, problems[0].K, workspace, (hipStream_t)stream) == hipSuccess ? FP6_OK
                                                                                                                    : FP6_ERR_HIP;
    }
    // one layer after another on the stream; they share the workspace in turn
    for (int i = 0; i < count; i++) {
        const int rc = linear_any(kE3M2, problems[i].X, M, problems[i].hi_plane, problems[i].lo_plane, problems[i].scales,
                                  problems[i].N, problems[i].K, 0, problems[i].Y, workspace, workspace_bytes, stream,
                                  FP6_VARIANT_AUTO, 0);
        if (rc != FP6_OK) return rc;
    }
    return FP6_OK;
}

int fp6_linear_plan(int format, int64_t M, int64_t N, int64_t K, int64_t block, int variant, int split_k,
                    fp6_plan_info* info)
{
    if (!info) return FP6_ERR_NULL;
    if (format != kE3M2 && format != kE3M1 && format != kE3M2H && format != kE3M2B) return FP6_ERR_VARIANT;
    if (M <= 0 || M > (int64_t)1 << 24 || !shape_ok(N, K) || block < 0) return FP6_ERR_SHAPE;
    LinearPlan p;
    if (!make_plan(format, M, N, K, block, variant, split_k, &p)) return FP6_ERR_VARIANT;
    const int64_t nblocks = N / FP6_TILE;
    info->variant = p.variant;
    info->split_k = p.split_k;
    info->block_m = p.block_m;
    info->waves = p.waves;
    info->depth = p.depth;
    info->half_tiles = p.half_tiles;
    info->meeting = p.split_k == 1 ? 0 : (p.pairwise ? 2 : 1);
    if (p.variant == FP6_VARIANT_DECODE) {
        // the grids of launch_decode_t / launch_decode_half_t
        info->width = 1;
        info->workgroups = p.half_tiles ? (nblocks * p.split_k + 7) / 8 * 16 : nblocks * p.split_k;
    } else {
        // the grid of launch_gemm_t
        info->width = p.gbn;
        const int64_t mblk = (M + p.block_m - 1) / p.block_m, nblk = (nblocks + p.gbn - 1) / p.gbn;
        info->workgroups = mblk * ((nblk * p.split_k + 7) / 8 * 8);
    }
    info->workspace_bytes = plan_workspace(p);
    return FP6_OK;
}

int fp6_linear_variant(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane,
                       const uint16_t* scales, int64_t N, int64_t K, uint16_t* Y, void* workspace,
                       size_t workspace_bytes, void* stream, int variant, int split_k)
{
    return linear_any(kE3M2, X, M, hi_plane, lo_plane, scales, N, K, 0, Y, workspace, workspace_bytes, stream, variant,
                      split_k);
}

int fp6_linear(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane, const uint16_t* scales,
               int64_t N, int64_t K, uint16_t* Y, void* workspace, size_t workspace_bytes, void* stream)
{
    return linear_any(kE3M2, X, M, hi_plane, lo_plane, scales, N, K, 0, Y, workspace, workspace_bytes, stream,
                      FP6_VARIANT_AUTO, 0);
}

int fp6_linear_static(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane, const uint16_t* scales,
                      int64_t N, int64_t K, uint16_t* Y, void* stream)
{
    if (!X || !hi_plane || !lo_plane || !scales || !Y) return FP6_ERR_NULL;
    if (M <= 0 || M > (int64_t)1 << 24 || !shape_ok(N, K)) return FP6_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(scales) || !aligned16(Y))
        return FP6_ERR_ALIGN;
    LinearPlan p;
    if (!make_plan(kE3M2, M, N, K, 0, FP6_VARIANT_AUTO, 0, &p)) return FP6_ERR_VARIANT;
    const size_t need = plan_workspace(p);
    if (need > (size_t)FP6_STATIC_SCRATCH_BYTES) return FP6_ERR_SCRATCH;
    void* ws = nullptr;
    if (need > 0) {
        ws = static_scratch((hipStream_t)stream);
        if (!ws) return FP6_ERR_HIP;
    }
    forget_earlier_errors();
    hipError_t e = (p.variant == FP6_VARIANT_DECODE)
                       ? launch_decode(p, X, M, hi_plane, lo_plane, scales, N, K, Y, ws, (hipStream_t)stream)
                       : launch_gemm(p, X, M, hi_plane, lo_plane, scales, N, K, Y, ws, (hipStream_t)stream);
    return e == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

int fp6_linear_fgq(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane, const uint16_t* scales,
                   int64_t N, int64_t K, int64_t block, uint16_t* Y, void* workspace, size_t workspace_bytes,
                   void* stream, int variant, int split_k)
{
    if (block <= 0) return FP6_ERR_SHAPE;
    return linear_any(kE3M2, X, M, hi_plane, lo_plane, scales, N, K, block, Y, workspace, workspace_bytes, stream, variant,
                      split_k);
}

// ---- FP6 in plane layout 2 (planes that merge into the operand of the hardware conversion)

int fp6_quantize_pack_v2(const uint16_t* W, int64_t N, int64_t K, void* hi_plane, void* lo_plane, uint16_t* scales,
                         void* stream)
{
    return quantize_pack_any(kE3M2H, W, N, K, 0, hi_plane, lo_plane, scales, stream);
}

int fp6_unpack_codes_v2(const void* hi_plane, const void* lo_plane, int64_t N, int64_t K, uint8_t* codes, void* stream)
{
    if (!hi_plane || !lo_plane || !codes) return FP6_ERR_NULL;
    if (!shape_ok(N, K)) return FP6_ERR_SHAPE;
    if (!aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(codes)) return FP6_ERR_ALIGN;
    forget_earlier_errors();
    return launch_unpack_codes(kE3M2H, hi_plane, lo_plane, N, K, codes, (hipStream_t)stream) == hipSuccess
               ? FP6_OK
               : FP6_ERR_HIP;
}

int fp6_dequantize_v2(const void* hi_plane, const void* lo_plane, const uint16_t* scales, int64_t N, int64_t K,
                      uint16_t* W_hat, void* stream)
{
    return dequantize_any(kE3M2H, hi_plane, lo_plane, scales, N, K, 0, W_hat, stream);
}

size_t fp6_linear_v2_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int split_k)
{
    return workspace_any(kE3M2H, M, N, K, 0, variant, split_k);
}

int fp6_linear_v2(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane, const uint16_t* scales,
                  int64_t N, int64_t K, uint16_t* Y, void* workspace, size_t workspace_bytes, void* stream, int variant,
                  int split_k)
{
    return linear_any(kE3M2H, X, M, hi_plane, lo_plane, scales, N, K, 0, Y, workspace, workspace_bytes, stream, variant,
                      split_k);
}

int fp6_linear_v2_bf16(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane, const uint16_t* scales,
                       int64_t N, int64_t K, uint16_t* Y, void* workspace, size_t workspace_bytes, void* stream,
                       int variant, int split_k)
{
    return linear_any(kE3M2B, X, M, hi_plane, lo_plane, scales, N, K, 0, Y, workspace, workspace_bytes, stream, variant,
                      split_k);
}

// ---- FP5 E3M1, "4+1"

int fp5_packed_sizes(int64_t N, int64_t K, size_t* hi_bytes, size_t* lo_bytes, size_t* scale_bytes)
{
    if (!shape_ok(N, K)) return FP6_ERR_SHAPE;
    if (hi_bytes) *hi_bytes = (size_t)(N * K / 2);
    if (lo_bytes) *lo_bytes = (size_t)(N * K / 8);
    if (scale_bytes) *scale_bytes = (size_t)(2 * N);
    return FP6_OK;
}

int fp5_quantize_pack(const uint16_t* W, int64_t N, int64_t K, void* hi_plane, void* lo_plane, uint16_t* scales,
                      void* stream)
{
    return quantize_pack_any(kE3M1, W, N, K, 0, hi_plane, lo_plane, scales, stream);
}

int fp5_unpack_codes(const void* hi_plane, const void* lo_plane, int64_t N, int64_t K, uint8_t* codes, void* stream)
{
    if (!hi_plane || !lo_plane || !codes) return FP6_ERR_NULL;
    if (!shape_ok(N, K)) return FP6_ERR_SHAPE;
    if (!aligned16(hi_plane) || !aligned16(lo_plane) || !aligned16(codes)) return FP6_ERR_ALIGN;
    forget_earlier_errors();
    return launch_unpack_codes(kE3M1, hi_plane, lo_plane, N, K, codes, (hipStream_t)stream) == hipSuccess
               ? FP6_OK
               : FP6_ERR_HIP;
}

int fp5_dequantize(const void* hi_plane, const void* lo_plane, const uint16_t* scales, int64_t N, int64_t K,
                   uint16_t* W_hat, void* stream)
{
    return dequantize_any(kE3M1, hi_plane, lo_plane, scales, N, K, 0, W_hat, stream);
}

size_t fp5_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int split_k)
{
    return workspace_any(kE3M1, M, N, K, 0, variant, split_k);
}

int fp5_linear(const uint16_t* X, int64_t M, const void* hi_plane, const void* lo_plane, const uint16_t* scales,
               int64_t N, int64_t K, uint16_t* Y, void* workspace, size_t workspace_bytes, void* stream, int variant,
               int split_k)
{
    return linear_any(kE3M1, X, M, hi_plane, lo_plane, scales, N, K, 0, Y, workspace, workspace_bytes, stream, variant,
                      split_k);
}

}  // extern "C"
