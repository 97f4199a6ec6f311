// Device-side building blocks shared by the gfx950 kernels: vector types, the
// 4+2 -> fp16 unpack (ZeroQuant(4+2) Sections 5.1-5.2) and the tile addressing of the
// packed planes (layout version 1, described in include/fp6_linear.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fp6_internal.hpp"

namespace fp6 {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTile = 64;             // tile edge in n and in k
constexpr int kHiTileBytes = 2048;    // 4-bit plane bytes per tile
constexpr int kLoTileBytes = 1024;    // 2-bit plane bytes per tile
constexpr int kHiTileVec = kHiTileBytes / 16;   // uint4 per tile
constexpr int kLoTileVec = kLoTileBytes / 16;
constexpr int kLo1TileBytes = 512;    // 1-bit plane bytes per tile (FP5): 8 bytes per lane
template <int FMT>
constexpr int kLoBytesOf = FMT == kE3M1 ? kLo1TileBytes : kLoTileBytes;

// bitwise select: mask bit 1 -> a, mask bit 0 -> b   (one v_bitop3_b32)
__device__ __forceinline__ uint32_t bit_select(uint32_t a, uint32_t b, uint32_t mask)
{
    return __builtin_amdgcn_bitop3_b32(a, b, mask, 0xE4);
}

// Raw packed data of one 64x64 tile as held by one lane: 64 weights.
struct TileRaw {
    u32x4 hi0;   // fragments 0..3: one dword per fragment (8 sign+exponent sub-numbers)
    u32x4 hi1;   // fragments 4..7
    u32x4 lo;    // FP6: dword d = the mantissa sub-numbers of fragments 2d and 2d+1
                 // FP5: dwords 0, 1 only; dword d = the mantissa bits of fragments 4d .. 4d+3
};

// Three coalesced 128-bit loads per lane.  The weight stream is read exactly once, so
// it is marked non-temporal to keep it from evicting X and the partial sums.
template <int FMT = kE3M2>
__device__ __forceinline__ TileRaw load_tile(const u32x4* __restrict__ hi, const u32x4* __restrict__ lo,
                                             size_t tile_index, int lane)
{
    TileRaw r;
    const u32x4* h = hi + tile_index * kHiTileVec + lane;
    r.hi0 = __builtin_nontemporal_load(h);
    r.hi1 = __builtin_nontemporal_load(h + 64);
    if (FMT != kE3M1) {
        r.lo = __builtin_nontemporal_load(lo + tile_index * kLoTileVec + lane);
    } else {
        const u32x2 l = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(lo) + tile_index * 64 + lane);
        r.lo = u32x4{l.x, l.y, 0u, 0u};
    }
    return r;
}

// f must be a compile-time constant after unrolling
__device__ __forceinline__ uint32_t tile_hi_dword(const TileRaw& r, int f)
{
    return (f < 4) ? r.hi0[f & 3] : r.hi1[f & 3];
}

__device__ __forceinline__ uint32_t tile_lo_dword(const TileRaw& r, int f) { return r.lo[f >> 1]; }

// Bias-shift unpack of one fragment (8 weights of one lane) into the four packed-fp16
// registers of an MFMA 16x16x32 operand.  Pure bit padding (Section 5.2, Eq. 5): the
// byte  s00eeemm  is the top byte of the fp16 pattern  s 00eee mm00000000, whose value is
// the FP6 value times 2^-12.  H = the fragment's dword of the 4-bit plane, L = its dword
// of the 2-bit plane already shifted right by 4*(f&1).
//   byte b of H: bit0 sign(grp0) bit1 sign(grp1) bits4..2 exp(grp0) bits7..5 exp(grp1)
//   byte b of L: bits1..0 mant(grp0) bits3..2 mant(grp1)
// Byte b carries element j = 2*(b&1) + (b>>1) of its group: bytes 0 and 2 become the low
// and high half of one operand register (elements 0,1), bytes 1 and 3 those of the next.
//
// How the padded sub-numbers become the fp16 MFMA operand:
//   kBiasShift   the method (Section 5.2, Eq. 5): nothing more is done; the operand is the FP6
//                value times 2^-12 and the 2^12 rides in the scale.
//   kIntRebias   ablation, the traditional dequantization of Section 5.2: integer arithmetic on
//                the exponent field (+12 = fp16 bias 15 - FP6 bias 3), FP6 subnormals special-cased.
//   kHalfMul     ablation: the padded pattern is multiplied by 2^12 in fp16, i.e. the
//                floating-point unit does the exponent arithmetic (subnormals included).
// The ablations produce the FP6 values themselves, and the row scale is applied without 2^12.
enum Dequant { kBiasShift = 0, kIntRebias = 1, kHalfMul = 2 };

// Four bytes  s g g e e e m m  ->  the top bytes of the fp16 numbers equal to the FP6 values:
// exponent field + 12 for normal numbers; the FP6 subnormals m/16 are normal numbers in fp16
// and are rebuilt case by case (0 -> 0, 1 -> 2^-4, 2 -> 2^-3, 3 -> 1.5 * 2^-3).
__device__ __forceinline__ uint32_t rebias_bytes(uint32_t u)
{
    u &= 0x9F9F9F9Fu;                                               // drop the don't-care bits
    const uint32_t e = u & 0x1C1C1C1Cu;
    const uint32_t nz = ((e | (e >> 1) | (e >> 2)) >> 2) & 0x01010101u;   // 1 in a byte: exponent field != 0
    const uint32_t normal = (nz << 8) - nz;                         // 0xFF in the bytes of normal numbers
    const uint32_t n = u + 0x30303030u;                             // 12 << 2 per byte; eee + 12 <= 19: no carry out
    const uint32_t m0 = u & 0x01010101u, m1 = (u >> 1) & 0x01010101u;
    const uint32_t any = m0 | m1, one = m0 & ~m1, three = m0 & m1;
    // subnormal bytes: sign | exponent 11 (m = 1) or 12 (m = 2, 3) | top mantissa bit (m = 3)
    const uint32_t sub = (u & 0x80808080u) | (any << 5) | (m1 << 4) | (one << 3) | (one << 2) | (three << 1);
    return bit_select(n, sub, normal);
}

template <int DQ = kBiasShift>
__device__ __forceinline__ half8 unpack_fragment(uint32_t H, uint32_t L)
{
    // s g g e e e m m per byte (g = don't-care bits removed by the final masks)
    uint32_t u0 = bit_select(H << 7, bit_select(H, L, 0x1C1C1C1Cu), 0x80808080u);
    uint32_t u1 = bit_select(H << 6, bit_select(H >> 3, L >> 2, 0x1C1C1C1Cu), 0x80808080u);
    if (DQ == kIntRebias) {
        u0 = rebias_bytes(u0);
        u1 = rebias_bytes(u1);
    }
    constexpr uint32_t kKeep = DQ == kIntRebias ? 0xFF00FF00u : 0x9F009F00u;
    u32x4 w;
    w.x = (u0 << 8) & kKeep;   // bytes 0,2 -> elements 0,1
    w.y = u0 & kKeep;          // bytes 1,3 -> elements 2,3
    w.z = (u1 << 8) & kKeep;   // elements 4,5
    w.w = u1 & kKeep;          // elements 6,7
    half8 h = __builtin_bit_cast(half8, w);
    if (DQ == kHalfMul) h *= (_Float16)4096.0f;
    return h;
}

// FP5 (E3M1): the same padding with one mantissa bit, which lands on bit 1 of the byte
// s00eeem0; bit 0 is cleared by the final mask.  M = the dword of the 1-bit plane that covers
// fragments 4*(f/4) .. +3: byte b holds, for fragment f, mant(grp0) at bit 2*(f%4) and
// mant(grp1) at bit 2*(f%4) + 1.
__device__ __forceinline__ half8 unpack_fragment_e3m1(uint32_t H, uint32_t M, int fq)
{
    const uint32_t L0 = fq ? M >> (2 * fq - 1) : M << 1;    // grp0 bit -> bit 1
    const uint32_t L1 = M >> (2 * fq);                      // grp1 bit -> bit 1
    uint32_t u0 = bit_select(H << 7, bit_select(H, L0, 0x1C1C1C1Cu), 0x80808080u);
    uint32_t u1 = bit_select(H << 6, bit_select(H >> 3, L1, 0x1C1C1C1Cu), 0x80808080u);
    u32x4 w;
    w.x = (u0 << 8) & 0x9E009E00u;
    w.y = u0 & 0x9E009E00u;
    w.z = (u1 << 8) & 0x9E009E00u;
    w.w = u1 & 0x9E009E00u;
    return __builtin_bit_cast(half8, w);
}

template <int DQ = kBiasShift, int FMT = kE3M2>
__device__ __forceinline__ half8 unpack_tile_fragment(const TileRaw& r, int f)
{
    if (FMT == kE3M1) return unpack_fragment_e3m1(tile_hi_dword(r, f), r.lo[f >> 2], f & 3);
    return unpack_fragment<DQ>(tile_hi_dword(r, f), tile_lo_dword(r, f) >> (4 * (f & 1)));
}

// ---- plane layout 2 (kE3M2H): merge in registers, convert in hardware ---------------------------
// A unit = the 32 weights a lane holds for one 32-wide k block of a tile: element i = 8t + e is
// element e (k = 8 * (lane/16) + e inside the block) of the 16-channel fragment t.  Written as a
// string of 192 bits, code i (s eee mm) sits at bits 6i .. 6i+5: that is the operand of
// v_cvt_scalef32_pk32_f16_bf6, which returns the 32 fp16 values - the four MFMA operands of the
// unit - exactly (probed on the GPU for every code; the scale operand contributes its exponent).
// The planes hold that string split by kind of bit.  Bit p of string dword j is a mantissa bit if
// (32j + p) % 6 < 2, else a sign/exponent bit.  The unit's two dwords of the 2-bit plane are the
// mantissa bits of string dwords 0..2 and 3..5, each at its own position (the three position sets
// are disjoint and fill a dword).  Its four dwords of the 4-bit plane are the sign/exponent bits of
// string dwords 0..3 at their own positions; the positions left over in them carry the
// sign/exponent bits of string dwords 4 and 5, which a shift by two puts in place.  Merging the
// planes back costs 11 logic operations per 32 weights.
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
typedef _Float16 half32 __attribute__((ext_vector_type(32)));
typedef __bf16 bf16x32 __attribute__((ext_vector_type(32)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr uint32_t kSE0 = 0x3CF3CF3Cu, kSE1 = 0xCF3CF3CFu, kSE2 = 0xF3CF3CF3u;   // sign/exponent positions of string dwords j % 3 = 0, 1, 2
constexpr uint32_t kFromA3 = 0xF0C30C30u;   // positions of string dword 5 that come from plane dword 3 (rotated)

__device__ __forceinline__ u32x6 merge_unit(u32x4 A, uint32_t B0, uint32_t B1)
{
    u32x6 T;
    T[0] = bit_select(A[0], B0, kSE0);
    T[1] = bit_select(A[1], B0, kSE1);
    T[2] = bit_select(A[2], B0, kSE2);
    T[3] = bit_select(A[3], B1, kSE0);
    T[4] = bit_select(bit_select(A[0], A[1] >> 2, ~kSE0), B1, kSE1);
    T[5] = bit_select(bit_select(__builtin_amdgcn_alignbit(A[3], A[3], 2), A[2] >> 2, kFromA3), B1, kSE2);
    return T;
}

// The four MFMA operands (fragments t = 0..3) of k block q of a tile.
template <int DQ, int FMT>
__device__ __forceinline__ void unpack_kblock(const TileRaw& r, int q, half8 (&w)[4])
{
    if (FMT == kE3M2H) {
        const u32x6 T = merge_unit(q ? r.hi1 : r.hi0, r.lo[2 * q], r.lo[2 * q + 1]);
        const half32 h = __builtin_amdgcn_cvt_scalef32_pk32_f16_bf6(T, 1.0f);
#pragma unroll
        for (int t = 0; t < 4; t++)
#pragma unroll
            for (int e = 0; e < 8; e++) w[t][e] = h[8 * t + e];
    } else if (FMT == kE3M2B) {
        // bf16 operands travel in the same 128-bit registers; only the MFMA and the final conversion know
        const u32x6 T = merge_unit(q ? r.hi1 : r.hi0, r.lo[2 * q], r.lo[2 * q + 1]);
        const bf16x32 h = __builtin_amdgcn_cvt_scalef32_pk32_bf16_bf6(T, 1.0f);
#pragma unroll
        for (int t = 0; t < 4; t++) {
            bf16x8 b;
#pragma unroll
            for (int e = 0; e < 8; e++) b[e] = h[8 * t + e];
            w[t] = __builtin_bit_cast(half8, b);
        }
    } else {
#pragma unroll
        for (int t = 0; t < 4; t++) w[t] = unpack_tile_fragment<DQ, FMT>(r, 2 * t + q);
    }
}

// What the accumulated sum has to be multiplied by besides the row scale: the 2^12 that the
// bias shift took out of every weight (Section 5.2, Eq. 5), or nothing.
template <int DQ, int FMT = kE3M2>
constexpr float kUnshift = (DQ == kBiasShift && !layout2(FMT)) ? 4096.0f : 1.0f;

// D(16x16, fp32) += A(16x32 fp16) * B(32x16 fp16).  Lane l supplies row l%16 of A and
// column l%16 of B for the eight k values of group l/16, and holds D[4*(l/16)+r][l%16].
__device__ __forceinline__ float4v mfma16x16x32(half8 a, half8 b, float4v c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// The same for the element type of the format: bf16 operands for kE3M2B (carried in half8 registers), fp16 otherwise.
template <int FMT>
__device__ __forceinline__ float4v mfma16x16x32_of(half8 a, half8 b, float4v c)
{
    if (FMT == kE3M2B)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Four results to the 16-bit output type of the format (round to nearest even), as they are stored.
template <int FMT>
__device__ __forceinline__ half4 to_out4(const float (&v)[4])
{
    if (FMT == kE3M2B) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        bf16x4 y;
#pragma unroll
        for (int r = 0; r < 4; r++) y[r] = (__bf16)v[r];
        return __builtin_bit_cast(half4, y);
    }
    half4 y;
#pragma unroll
    for (int r = 0; r < 4; r++) y[r] = (_Float16)v[r];
    return y;
}

}  // namespace fp6
