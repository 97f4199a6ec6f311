// Meeting point for workgroups that each hold the partial sum of one K-slice of the
// same output tile.  Every workgroup stores its partial sums, then calls arrive_last();
// exactly one of them - the one whose arrival completes the count - gets `true`, and
// may then read all slices.  Nobody waits: there is no spinning, so the grid always
// drains.  The counter is left at zero for the next launch.
#pragma once

#include "fp6_common.hpp"

namespace fp6 {

// Must be called by every thread of the workgroup (it contains barriers).
__device__ __forceinline__ bool arrive_last(uint32_t* counter, uint32_t expected)
{
    __shared__ uint32_t s_last;
    __threadfence();   // release: this thread's partial sums are visible device-wide
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t last = (old == expected - 1u) ? 1u : 0u;
        if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = last;
    }
    __syncthreads();
    const bool last = s_last != 0u;
    if (last) __threadfence();   // acquire: the other workgroups' partial sums are visible
    return last;
}

// Partial sums written by other workgroups during this launch; only valid after
// arrive_last() returned true (its acquire fence drops stale cache lines).
__device__ __forceinline__ float4v load_partial(const float4v* p)
{
    return *p;
}

}  // namespace fp6
