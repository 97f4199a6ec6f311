// Meeting point for workgroups that each hold the partial sum of one K-slice of the
// same output tile.  Every workgroup stores its partial sums, then calls arrive_last();
// exactly one of them - the one whose arrival completes the count - gets `true`, and
// may then read all slices.  Nobody waits: there is no spinning, so the grid always
// drains.  The counter is left at zero for the next launch.
//
// The compute dies of the GPU each have their own L2.  A device-wide release/acquire
// fence would write back and invalidate that whole cache (microseconds per workgroup),
// so the exchange avoids it: partial sums are stored and loaded with the agent-coherent
// cache policy (sc1: written through to / read from the point where all dies agree),
// the arrival counter is an agent-scope atomic, and the only ordering needed is that a
// workgroup's stores have completed (vmcnt == 0) before its arrival is counted.
#pragma once

#include "fp6_common.hpp"

namespace fp6 {

constexpr int kAgentCoherent = 1 << 4;   // sc1 bit of the buffer-instruction cache policy

// Window onto `bytes` bytes of partial sums starting at base (wave-uniform).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t partial_window(float4v* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, bytes, 0x00020000);
}

__device__ __forceinline__ void store_partial(__amdgpu_buffer_rsrc_t win, uint32_t index, float4v v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), win, index * 16u, 0, kAgentCoherent);
}

// Only meaningful after arrive_last() returned true.
__device__ __forceinline__ float4v load_partial(__amdgpu_buffer_rsrc_t win, uint32_t index)
{
    return __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(win, index * 16u, 0, kAgentCoherent));
}

// Must be called by every thread of the workgroup (it contains barriers).
__device__ __forceinline__ bool arrive_last(uint32_t* counter, uint32_t expected)
{
    __shared__ uint32_t s_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partial sums have been written through
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t last = (old == expected - 1u) ? 1u : 0u;
        if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = last;
    }
    __syncthreads();
    return s_last != 0u;
}

}  // namespace fp6
