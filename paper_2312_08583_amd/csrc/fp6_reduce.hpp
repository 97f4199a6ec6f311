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

// ---- Pairwise meeting: a second way for K-slices to be added, for small partial sums.
//
// Two parties meet in a 64-bit slot that is zero when idle.  Each swaps its two fp32
// values (encoded so that they are never zero) into the slot with one agent-scope atomic
// exchange.  Whoever gets zero back came first and is done: its values now wait in the
// slot.  Whoever gets values back came second: it adds them to its own, writes zero back
// and carries the sum on.  One memory round trip, no barrier and no waiting; which party
// carries on depends on timing, the sum does not (a + b == b + a in IEEE arithmetic).
// More than two slices meet in a binary tree over the slice index, so the association
// order ((s0+s1)+(s2+s3))+... is fixed as well.
struct Pair {
    float a, b;
};

__device__ __forceinline__ uint32_t nonzero_code(float v)
{
    uint32_t w = ~__builtin_bit_cast(uint32_t, v);
    return w ? w : ~0x7FC00000u;      // the all-ones NaN pattern is posted as the default NaN
}
__device__ __forceinline__ float from_code(uint32_t w) { return __builtin_bit_cast(float, ~w); }

// Returns true if this caller carries the sum (then `v` holds it), false if it is done.
__device__ __forceinline__ bool meet_pair(unsigned long long* slot, Pair& v)
{
    const unsigned long long mine = ((unsigned long long)nonzero_code(v.b) << 32) | nonzero_code(v.a);
    const unsigned long long other = __hip_atomic_exchange(slot, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (other == 0ull) return false;
    __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.a += from_code((uint32_t)other);
    v.b += from_code((uint32_t)(other >> 32));
    return true;
}

// Tree over `count` slices; `index` is this caller's slice.  `slots` points at this
// value pair's first slot; consecutive tree nodes are `node_stride` slots apart and
// count - 1 of them are used.  Returns true for exactly one of the `count` callers,
// with the total in `v`.
__device__ __forceinline__ bool meet_tree(unsigned long long* slots, size_t node_stride, int index, int count, Pair& v)
{
    int node0 = 0;
    while (count > 1) {
        if ((index ^ 1) < count) {
            if (!meet_pair(slots + (size_t)(node0 + (index >> 1)) * node_stride, v)) return false;
        }
        node0 += count >> 1;
        index >>= 1;
        count = (count + 1) >> 1;
    }
    return true;
}

}  // namespace fp6
