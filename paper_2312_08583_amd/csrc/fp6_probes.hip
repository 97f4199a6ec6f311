// Measurement aids: what this chip sustains on the two resources that bound fp6_linear, measured
// by kernels that do nothing else.  A benchmark prints these ceilings beside the published peaks,
// so a fraction of the nominal peak can be read against what a plain kernel reaches on the same box.
//
//   read probe : every workgroup streams its share of a buffer with 128-bit non-temporal loads,
//                folds the words into one value and writes it (the fold keeps the loads alive).
//   MFMA probe : every wavefront holds four A and two B fragments in registers and issues
//                v_mfma_f32_16x16x32_f16 on eight independent accumulators in a loop, the register
//                tile of a dense fp16 GEMM without its loads.  Operands are either pseudo-random
//                fp16 in (-1, 1) or zeros: the matrix pipes draw less power on zeros, and the clock
//                the chip holds under load depends on it.  A third form follows every MFMA with two
//                independent integer vector instructions (v_perm_b32, v_xor_b32), the ratio of the tiled
//                kernel's loop, where the 4+2-bit unpack shares the vector issue port with the MFMAs.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fp6_linear.h"
#include "fp6_common.hpp"

namespace fp6 {

__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4* __restrict__ buf, size_t n16, uint32_t* __restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(buf + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // one word per wavefront leaves the kernel
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0) sink[(size_t)blockIdx.x * 4 + (threadIdx.x >> 6)] = acc;
}

__device__ __forceinline__ half8 probe_fragment(uint32_t seed, bool random)
{
    half8 f;
    for (int i = 0; i < 8; ++i) {
        seed = seed * 1664525u + 1013904223u;
        // 11 random bits -> a value in (-1, 1) with a full fp16 significand
        const float v = ((float)((seed >> 12) & 2047) - 1023.5f) * (1.0f / 1024.0f);
        f[i] = random ? (_Float16)v : (_Float16)0.0f;
    }
    return f;
}

typedef float float16v __attribute__((ext_vector_type(16)));

// WIDE = false: v_mfma_f32_16x16x32_f16 (4 accumulator registers); true: v_mfma_f32_32x32x16_f16 (16).
// Both do 16 * 16 * 32 * 2 * (WIDE ? 2 : 1) flop per instruction.
// MIX (with WIDE = false): a v_perm_b32 and a v_xor_b32 on registers of their own behind every MFMA.
template <bool WIDE, bool MIX = false>
__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(int iters, int random, float* __restrict__ sink)
{
    const uint32_t id = blockIdx.x * 256 + threadIdx.x;
    half8 a[4], b[2];
    for (int i = 0; i < 4; ++i) a[i] = probe_fragment(id * 8 + i + 1, random != 0);
    for (int j = 0; j < 2; ++j) b[j] = probe_fragment(id * 8 + 5 + j, random != 0);
    float s = 0.0f;
    if constexpr (MIX) {
        float4v acc[4][2] = {};
        uint32_t v[8];
        for (int i = 0; i < 8; ++i) v[i] = id * 2654435761u + i;
#pragma unroll 1
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[i][j] = mfma16x16x32(a[i], b[j], acc[i][j]);
                    const int r = i * 2 + j;
                    v[r] = __builtin_amdgcn_perm(v[r], v[(r + 1) & 7], 0x02010003u) ^ 0x5a5a5a5au;
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA, then two vector instructions
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                }
        }
        uint32_t x = 0;
        for (int i = 0; i < 8; ++i) x ^= v[i];
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 2; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
        s += (float)(x & 1u);
    } else if constexpr (WIDE) {
        float16v acc[4][2] = {};
#pragma unroll 1
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 2; ++j)
                for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    } else {
        float4v acc[4][2] = {};
#pragma unroll 1
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma16x16x32(a[i], b[j], acc[i][j]);
        }
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 2; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    }
    sink[id] = s;
}

}  // namespace fp6

extern "C" {

int fp6_probe_read(const void* buf, size_t bytes, int workgroups, void* sink, size_t sink_bytes, void* stream)
{
    if (!buf || !sink) return FP6_ERR_NULL;
    if (((uintptr_t)buf & 15) || ((uintptr_t)sink & 3)) return FP6_ERR_ALIGN;
    if (bytes < 16 || workgroups < 1 || workgroups > (1 << 20)) return FP6_ERR_SHAPE;
    if (sink_bytes < (size_t)workgroups * 16) return FP6_ERR_WORKSPACE;
    (void)hipGetLastError();      // drop an earlier call's error: the status below is this launch's
    hipLaunchKernelGGL(fp6::read_probe_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream,
                       (const fp6::u32x4*)buf, bytes / 16, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

int fp6_probe_mfma(int workgroups, int iters, int random_operands, int form, void* sink, size_t sink_bytes, void* stream)
{
    if (!sink) return FP6_ERR_NULL;
    if (form < 0 || form > 2) return FP6_ERR_VARIANT;
    if ((uintptr_t)sink & 3) return FP6_ERR_ALIGN;
    if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24)) return FP6_ERR_SHAPE;
    if (sink_bytes < (size_t)workgroups * 256 * sizeof(float)) return FP6_ERR_WORKSPACE;
    (void)hipGetLastError();
    if (form == 2)
        hipLaunchKernelGGL((fp6::mfma_probe_kernel<false, true>), dim3(workgroups), dim3(256), 0, (hipStream_t)stream,
                           iters, random_operands, (float*)sink);
    else if (form == 1)
        hipLaunchKernelGGL(fp6::mfma_probe_kernel<true>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream,
                           iters, random_operands, (float*)sink);
    else
        hipLaunchKernelGGL(fp6::mfma_probe_kernel<false>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream,
                           iters, random_operands, (float*)sink);
    return hipGetLastError() == hipSuccess ? FP6_OK : FP6_ERR_HIP;
}

}  // extern "C"
