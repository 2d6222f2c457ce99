// Cross-workgroup synchronisation that needs no zero-initialised memory.
//
// The workspace a caller hands in has undefined contents, and the library may
// not spend a launch on clearing it.  Every call therefore draws a fresh
// 40-bit epoch on the host; counters and flags in the workspace carry the
// epoch in their upper bits, and a word whose epoch differs from the current
// call's is treated as "not yet touched by this call".
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kEpochShift = 24;                              // low 24 bits: arrival count
constexpr unsigned long long kCountMask = (1ull << kEpochShift) - 1;

// Arrival ticket 0..n-1 of the calling workgroup for this epoch.  Stale contents
// (another epoch, or garbage) count as zero arrivals.
__device__ __forceinline__ uint32_t ticket_take(unsigned long long *ctr, unsigned long long epoch)
{
    unsigned long long old = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
        const unsigned long long nw = ((old >> kEpochShift) == epoch) ? old + 1 : ((epoch << kEpochShift) | 1ull);
        if (__hip_atomic_compare_exchange_strong(ctr, &old, nw, __ATOMIC_ACQ_REL, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT))
            return (uint32_t)(nw & kCountMask) - 1u;
    }
}

__device__ __forceinline__ void flag_publish(unsigned long long *flag, unsigned long long epoch)
{
    __hip_atomic_store(flag, epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Spins until *flag == epoch, at most `spin_limit` polls; returns false on
// timeout so that every wave still reaches the end of the kernel.
__device__ __forceinline__ bool flag_wait(const unsigned long long *flag, unsigned long long epoch, uint32_t spin_limit)
{
    for (uint32_t i = 0; i < spin_limit; ++i) {
        if (__hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == epoch) return true;
        __builtin_amdgcn_s_sleep(2);
    }
    return false;
}

}  // namespace sv
