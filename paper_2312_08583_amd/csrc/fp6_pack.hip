// Offline quantizer / packer (ZeroQuant(4+2) Section 4 Eq. 3, Section 5.1) and the two
// plane-reading test utilities, for gfx950.
#include "fp6_common.hpp"
#include "fp6_internal.hpp"

namespace fp6 {

// ------------------------------------------------------------------ scales
// S = RNE_fp16(max |w| / 28) over one block of `block` consecutive elements of a row
// (Section 4, Eq. 3; block == K is the row-wise scheme, smaller blocks the fine-grained
// one of Section 3).  Scale (n, g) is stored at scales[g * N + n]: block-major, so that the
// scales of neighbouring output channels are neighbours in memory.
// |w| of finite fp16 orders like its 15 magnitude bits, so the maximum is taken on
// integers.  The quotient is one IEEE fp32 division followed by one fp32->fp16 rounding;
// a double rounding cannot occur because amax/28 is either exact in fp16 or at least
// 2^-14 (relative) away from every fp16 midpoint.
__global__ __launch_bounds__(256) void block_scale_kernel(const uint16_t* __restrict__ W, int64_t N, int64_t K,
                                                           int64_t block, float fmax, uint16_t* __restrict__ scales)
{
    const int64_t G = K / block;
    const int64_t n = blockIdx.x / G, g = blockIdx.x % G;
    const uint4* row = reinterpret_cast<const uint4*>(W + n * K + g * block);
    const int64_t nvec = block / 8;
    uint32_t amax = 0;
    for (int64_t v = threadIdx.x; v < nvec; v += blockDim.x) {
        uint4 d = row[v];
        uint32_t w[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            amax = max(amax, w[i] & 0x7FFFu);
            amax = max(amax, (w[i] >> 16) & 0x7FFFu);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, off, 64));
    __shared__ uint32_t s_max[4];
    if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = amax;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (unsigned w = 1; w < blockDim.x / 64; w++) amax = max(amax, s_max[w]);
        float a = (float)__builtin_bit_cast(_Float16, (uint16_t)amax);
        _Float16 S = (_Float16)(a / fmax);      // 28 for E3M2, 24 for E3M1 (the format's largest magnitude)
        scales[g * N + n] = __builtin_bit_cast(uint16_t, S);
    }
}

// Round-to-nearest E3M2 code of w / S (ties to the even code, saturating at 28).
// q = |w|/S is one correctly rounded fp32 division: a quotient that is not exactly a
// grid midpoint is at least 2^-17 (relative) away from it, far more than the 2^-24 the
// division can move it, and an exact midpoint divides exactly - so rounding q decides
// exactly as rounding the real quotient would.  The rounding itself works on the bit pattern
// of q.  From 0.25 up the code is the top of that pattern: exponent field and the first MB
// mantissa bits, rounded to nearest even in place (half a unit minus one, plus the last kept
// bit, is added below them; a carry runs into the exponent as it should), re-biased from 127
// to 3.  Below 0.25 the codes count multiples of 2^-(2+MB): adding 2^(21-MB) makes the fp32
// addition round q to that spacing (to nearest even) and leaves the count in the low bits.
// MB = mantissa bits: 2 for E3M2 (largest value 28), 1 for E3M1 (24).
template <int MB = 2>
__device__ __forceinline__ uint32_t e3m2_code(uint16_t wbits, float S)
{
    const uint32_t sign = (wbits >> 15) << (3 + MB);
    if (S == 0.0f) return sign;
    const float a = (float)__builtin_bit_cast(_Float16, (uint16_t)(wbits & 0x7FFFu));
    const float q = fminf(a / S, MB == 2 ? 28.0f : 24.0f);
    constexpr int kDrop = 23 - MB;                               // mantissa bits of q below the code
    const uint32_t b = __builtin_bit_cast(uint32_t, q);
    const uint32_t top = (b + ((1u << (kDrop - 1)) - 1u) + ((b >> kDrop) & 1u)) >> kDrop;
    const uint32_t normal = top - (124u << MB);                  // (exponent + 3) << MB | mantissa
    const float t = q + (float)(1u << (21 - MB));                // spacing 2^-(2+MB) in that binade
    const uint32_t sub = __builtin_bit_cast(uint32_t, t) & 7u;   // 0 .. 2^MB (the last one is 0.25 itself)
    return sign | (q < 0.25f ? sub : normal);
}

// One thread = one lane slot of one tile (64 weights): reads its eight 8-element runs of
// W, quantizes them, and writes its 32 + 16 bytes of the two planes.
template <int FMT>
__global__ __launch_bounds__(256) void quantize_pack_kernel(const uint16_t* __restrict__ W, int64_t N, int64_t K,
                                                             int64_t block, const uint16_t* __restrict__ scales,
                                                             uint4* __restrict__ hi, uint4* __restrict__ lo)
{
    const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t tile = slot >> 6;
    const int lane = (int)(slot & 63);
    const int64_t ktiles = K / kTile;
    if (tile >= (N / kTile) * ktiles) return;
    const int64_t nb = tile / ktiles, kb = tile % ktiles;
    const int i = lane & 15, g = lane >> 4;

    uint32_t hiw[8], low[4] = {0, 0, 0, 0};
    uint32_t T[2][7] = {{0, 0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0, 0}};     // layout 2: the two units' bit strings (+ spill-over dword)
#pragma unroll
    for (int f = 0; f < 8; f++) {
        const int64_t n = nb * kTile + (f >> 1) * 16 + i;
        const int64_t k = kb * kTile + (f & 1) * 32 + g * 8;
        const float S = (float)__builtin_bit_cast(_Float16, scales[(k / block) * N + n]);
        uint4 d = *reinterpret_cast<const uint4*>(W + n * K + k);
        uint32_t w2[4] = {d.x, d.y, d.z, d.w};
        uint32_t h = 0, l = 0;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            uint16_t wb = (uint16_t)((e & 1) ? (w2[e >> 1] >> 16) : (w2[e >> 1] & 0xFFFFu));
            if (FMT == kE3M2H) {
                // code i = 8t + e of unit q = f & 1 at bits 6i .. 6i+5 of the unit's string
                const uint32_t c = e3m2_code<2>(wb, S);
                const int bit = 6 * (8 * (f >> 1) + e);
                T[f & 1][bit >> 5] |= c << (bit & 31);
                if ((bit & 31) > 26) T[f & 1][(bit >> 5) + 1] |= c >> (32 - (bit & 31));
                continue;
            }
            constexpr int MB = FMT == kE3M1 ? 1 : 2;
            uint32_t c = e3m2_code<MB>(wb, S);
            const int grp = e >> 2, j = e & 3;
            const int b = 2 * (j & 1) + (j >> 1);
            const uint32_t s = c >> (3 + MB), ex = (c >> MB) & 7, m = c & ((1u << MB) - 1u);
            h |= (s << grp | ex << (2 + 3 * grp)) << (8 * b);
            l |= (m << (MB * grp)) << (8 * b);
        }
        hiw[f] = h;
        if (FMT == kE3M2) low[f >> 1] |= l << (4 * (f & 1));
        else if (FMT == kE3M1) low[f >> 2] |= l << (2 * (f & 3));
    }
    if (FMT == kE3M2H) {
        // split each string by kind of bit (the inverse of merge_unit)
#pragma unroll
        for (int q = 0; q < 2; q++) {
            const uint32_t* t = T[q];
            low[2 * q] = (t[0] & ~kSE0) | (t[1] & ~kSE1) | (t[2] & ~kSE2);
            low[2 * q + 1] = (t[3] & ~kSE0) | (t[4] & ~kSE1) | (t[5] & ~kSE2);
            hiw[4 * q + 0] = (t[0] & kSE0) | (t[4] & ~kSE0);
            hiw[4 * q + 1] = (t[1] & kSE1) | ((t[4] & 0x0C30C30Cu) << 2);
            hiw[4 * q + 2] = (t[2] & kSE2) | ((t[5] & 0x030C30C3u) << 2);
            const uint32_t r5 = t[5] & kFromA3;
            hiw[4 * q + 3] = (t[3] & kSE0) | (r5 << 2) | (r5 >> 30);
        }
    }
    uint4* hp = hi + tile * kHiTileVec + lane;
    hp[0] = make_uint4(hiw[0], hiw[1], hiw[2], hiw[3]);
    hp[64] = make_uint4(hiw[4], hiw[5], hiw[6], hiw[7]);
    if (FMT != kE3M1) lo[tile * kLoTileVec + lane] = make_uint4(low[0], low[1], low[2], low[3]);
    else reinterpret_cast<uint2*>(lo)[tile * 64 + lane] = make_uint2(low[0], low[1]);
}

// ------------------------------------------------------------------ plane readers
// code of element e (0..7) of a fragment, from its two dwords (L already shifted by 4*(f&1))
// MB = 2: L = the fragment's dword of the 2-bit plane shifted right by 4*(f&1); code s eee mm.
// MB = 1: L = its dword of the 1-bit plane shifted right by 2*(f&3); code s eee m.
template <int MB = 2>
__device__ __forceinline__ uint32_t fragment_code(uint32_t H, uint32_t L, int e)
{
    const int grp = e >> 2, j = e & 3;
    const int b = 2 * (j & 1) + (j >> 1);
    const uint32_t hb = (H >> (8 * b)) & 0xFF, lb = (L >> (8 * b)) & 0xFF;
    const uint32_t s = (hb >> grp) & 1, ex = (hb >> (2 + 3 * grp)) & 7, m = (lb >> (MB * grp)) & ((1u << MB) - 1u);
    return s << (3 + MB) | ex << MB | m;
}

// the fragment's plane dwords as fragment_code wants them
template <int FMT>
__device__ __forceinline__ uint32_t fragment_lo(const TileRaw& r, int f)
{
    return FMT == kE3M2 ? tile_lo_dword(r, f) >> (4 * (f & 1)) : r.lo[f >> 2] >> (2 * (f & 3));
}

// code of element e of fragment f of a tile, any layout (f, e compile-time constants after unrolling)
template <int FMT>
__device__ __forceinline__ uint32_t tile_code(const TileRaw& r, int f, int e)
{
    if (FMT == kE3M2H) {
        const int q = f & 1, bit = 6 * (8 * (f >> 1) + e);
        const u32x6 T = merge_unit(q ? r.hi1 : r.hi0, r.lo[2 * q], r.lo[2 * q + 1]);
        uint32_t c = T[bit >> 5] >> (bit & 31);
        if ((bit & 31) > 26) c |= T[(bit >> 5) + 1] << (32 - (bit & 31));
        return c & 63u;
    }
    return fragment_code<FMT == kE3M1 ? 1 : 2>(tile_hi_dword(r, f), fragment_lo<FMT>(r, f), e);
}

template <int FMT>
__global__ __launch_bounds__(256) void unpack_codes_kernel(const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
                                                            int64_t N, int64_t K, uint8_t* __restrict__ codes)
{
    const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t tile = slot >> 6;
    const int lane = (int)(slot & 63);
    const int64_t ktiles = K / kTile;
    if (tile >= (N / kTile) * ktiles) return;
    const int64_t nb = tile / ktiles, kb = tile % ktiles;
    const int i = lane & 15, g = lane >> 4;
    TileRaw r = load_tile<FMT>(hi, lo, (size_t)tile, lane);
#pragma unroll
    for (int f = 0; f < 8; f++) {
        const int64_t n = nb * kTile + (f >> 1) * 16 + i;
        const int64_t k = kb * kTile + (f & 1) * 32 + g * 8;
        uint32_t c0 = 0, c1 = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            c0 |= tile_code<FMT>(r, f, e) << (8 * e);
            c1 |= tile_code<FMT>(r, f, 4 + e) << (8 * e);
        }
        *reinterpret_cast<uint2*>(codes + n * K + k) = make_uint2(c0, c1);
    }
}

// W_hat = RNE_fp16(S * value(code)): the fp32 product of an 11-bit and a 3-bit
// significand is exact, so the only rounding is the conversion to fp16.
template <int FMT>
__global__ __launch_bounds__(256) void dequantize_kernel(const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
                                                          const uint16_t* __restrict__ scales, int64_t N, int64_t K,
                                                          int64_t block, uint16_t* __restrict__ W_hat)
{
    const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t tile = slot >> 6;
    const int lane = (int)(slot & 63);
    const int64_t ktiles = K / kTile;
    if (tile >= (N / kTile) * ktiles) return;
    const int64_t nb = tile / ktiles, kb = tile % ktiles;
    const int i = lane & 15, g = lane >> 4;
    constexpr int MB = FMT == kE3M1 ? 1 : 2;
    TileRaw r = load_tile<FMT>(hi, lo, (size_t)tile, lane);
#pragma unroll
    for (int f = 0; f < 8; f++) {
        const int64_t n = nb * kTile + (f >> 1) * 16 + i;
        const int64_t k = kb * kTile + (f & 1) * 32 + g * 8;
        const float S = (float)__builtin_bit_cast(_Float16, scales[(k / block) * N + n]);
        uint32_t out[4];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const uint32_t c = tile_code<FMT>(r, f, e);
            const uint32_t ex = (c >> MB) & 7, m = (c & ((1u << MB) - 1u)) << (2 - MB);   // mantissa as quarters
            // value = m/16 (subnormal) or (4+m) * 2^(ex-5)
            float mag = ex ? (float)((4 + m) << (ex - 1)) * 0.0625f : (float)m * 0.0625f;
            _Float16 hval = (_Float16)(S * mag);
            uint32_t hb = __builtin_bit_cast(uint16_t, hval) | ((c >> (3 + MB)) << 15);
            if (e & 1) out[e >> 1] |= hb << 16; else out[e >> 1] = hb;
        }
        *reinterpret_cast<uint4*>(W_hat + n * K + k) = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

// ------------------------------------------------------------------ launchers
static inline unsigned slot_blocks(int64_t N, int64_t K) { return (unsigned)(((N / kTile) * (K / kTile) * 64 + 255) / 256); }

hipError_t launch_quantize_pack(int format, const uint16_t* W, int64_t N, int64_t K, int64_t block, void* hi, void* lo,
                                uint16_t* scales, hipStream_t stream)
{
    hipLaunchKernelGGL(block_scale_kernel, dim3((unsigned)(N * (K / block))), dim3(block >= 2048 ? 256 : 64), 0, stream,
                       W, N, K, block, format == kE3M1 ? 24.0f : 28.0f, scales);
    if (format == kE3M2)
        hipLaunchKernelGGL(quantize_pack_kernel<kE3M2>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, W, N, K, block,
                           (const uint16_t*)scales, (uint4*)hi, (uint4*)lo);
    else if (format == kE3M2H)
        hipLaunchKernelGGL(quantize_pack_kernel<kE3M2H>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, W, N, K, block,
                           (const uint16_t*)scales, (uint4*)hi, (uint4*)lo);
    else
        hipLaunchKernelGGL(quantize_pack_kernel<kE3M1>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, W, N, K, block,
                           (const uint16_t*)scales, (uint4*)hi, (uint4*)lo);
    return hipGetLastError();
}

hipError_t launch_unpack_codes(int format, const void* hi, const void* lo, int64_t N, int64_t K, uint8_t* codes,
                               hipStream_t stream)
{
    if (format == kE3M2)
        hipLaunchKernelGGL(unpack_codes_kernel<kE3M2>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, (const u32x4*)hi,
                           (const u32x4*)lo, N, K, codes);
    else if (format == kE3M2H)
        hipLaunchKernelGGL(unpack_codes_kernel<kE3M2H>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, (const u32x4*)hi,
                           (const u32x4*)lo, N, K, codes);
    else
        hipLaunchKernelGGL(unpack_codes_kernel<kE3M1>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, (const u32x4*)hi,
                           (const u32x4*)lo, N, K, codes);
    return hipGetLastError();
}

hipError_t launch_dequantize(int format, const void* hi, const void* lo, const uint16_t* scales, int64_t N, int64_t K,
                             int64_t block, uint16_t* W_hat, hipStream_t stream)
{
    if (format == kE3M2)
        hipLaunchKernelGGL(dequantize_kernel<kE3M2>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, (const u32x4*)hi,
                           (const u32x4*)lo, scales, N, K, block, W_hat);
    else if (format == kE3M2H)
        hipLaunchKernelGGL(dequantize_kernel<kE3M2H>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, (const u32x4*)hi,
                           (const u32x4*)lo, scales, N, K, block, W_hat);
    else
        hipLaunchKernelGGL(dequantize_kernel<kE3M1>, dim3(slot_blocks(N, K)), dim3(256), 0, stream, (const u32x4*)hi,
                           (const u32x4*)lo, scales, N, K, block, W_hat);
    return hipGetLastError();
}

}  // namespace fp6
