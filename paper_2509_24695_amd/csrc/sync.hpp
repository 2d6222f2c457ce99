// Cross-workgroup synchronisation that needs no zero-initialised memory.
//
// Data that crosses workgroups inside one kernel (partial states, the updated
// state of the fused block step) is written and read with device-coherent
// accesses, and a wave waits for its own coherent stores to be performed before
// the workgroup signals; the signals themselves are relaxed atomics.
//
// The workspace a caller hands in has undefined contents, and the library may
// not spend a launch on clearing it.  Every call therefore draws a fresh
// 40-bit epoch on the host; counters and flags in the workspace carry the
// epoch in their upper bits, and a word whose epoch differs from the current
// call's is treated as "not yet touched by this call".
#pragma once

#include "common.hpp"

namespace sv {

// Device-coherent 8-byte accesses (relaxed atomics at agent scope).  On a
// multi-die GPU each die's L2 is private: such accesses are performed at the
// level all dies share, so data exchanged between workgroups of one kernel
// never needs a whole-cache write-back or invalidate.
__device__ __forceinline__ void store_coherent(float *p, f32x2 v) {
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ f32x2 load_coherent(const float *p) {
    return __builtin_bit_cast(f32x2, __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p),
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ float load_coherent1(const float *p) {
    return __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const unsigned int *>(p), __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT));
}
// All of this wave's earlier coherent stores have been performed once this
// returns; also keeps the compiler from moving memory operations across it.
__device__ __forceinline__ void coherent_stores_done() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

constexpr int kEpochShift = 24;                              // low 24 bits: arrival count
constexpr unsigned long long kCountMask = (1ull << kEpochShift) - 1;

// Arrival ticket 0..n-1 of the calling workgroup for this epoch.  Stale contents
// (another epoch, or garbage) count as zero arrivals.
__device__ __forceinline__ uint32_t ticket_take(unsigned long long *ctr, unsigned long long epoch)
{
    unsigned long long old = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
        const unsigned long long nw = ((old >> kEpochShift) == epoch) ? old + 1 : ((epoch << kEpochShift) | 1ull);
        if (__hip_atomic_compare_exchange_strong(ctr, &old, nw, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT))
            return (uint32_t)(nw & kCountMask) - 1u;
    }
}

__device__ __forceinline__ void flag_publish(unsigned long long *flag, unsigned long long epoch)
{
    __hip_atomic_store(flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Spins until *flag == epoch, at most `spin_limit` polls; returns false on
// timeout so that every wave still reaches the end of the kernel.
__device__ __forceinline__ bool flag_wait(const unsigned long long *flag, unsigned long long epoch, uint32_t spin_limit)
{
    for (uint32_t i = 0; i < spin_limit; ++i) {
        if (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == epoch) return true;
        __builtin_amdgcn_s_sleep(2);
    }
    return false;
}

}  // namespace sv
