// Cross-workgroup synchronisation that needs no zero-initialised memory.
//
// Data that crosses workgroups inside one kernel (partial states, the updated
// state of the fused block step) is written and read with device-coherent
// accesses, and a wave waits for its own coherent stores to be performed before
// the workgroup signals; the signals themselves are relaxed atomics.
//
// The workspace a caller hands in has undefined contents, and the library may
// not spend a launch on clearing it.  Every call therefore draws a fresh
// epoch on the host; a flag word in the workspace that does not hold the
// current call's epoch means "not yet published in this call".
#pragma once

#include "common.hpp"

namespace sv {

// Device-coherent 8-byte accesses (relaxed atomics at agent scope).  On a
// multi-die GPU each die's L2 is private: such accesses are performed at the
// level all dies share, so data exchanged between workgroups of one kernel
// never needs a whole-cache write-back or invalidate.
// LOCAL: every workgroup that will read the value runs on the writer's die (they share its L2), so a
// plain store, which ends in that L2, is enough: it is acknowledged without the trip to memory, and the
// readers' coherent loads find it there.
template <bool LOCAL = false>
__device__ __forceinline__ void store_coherent(float *p, f32x2 v) {
    if (LOCAL) *reinterpret_cast<f32x2 *>(p) = v;
    else __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Device-coherent 4-byte store through a buffer resource: the same cache policy as store_coherent,
// and byte offsets at or past the resource's size are dropped.
__device__ __forceinline__ void store_coherent4(rsrc_t r, uint32_t off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r, off, 0, 16 /* sc1 */);
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

// Epoch-tagged arrival flags.  A workgroup publishes by storing the call's
// epoch into its own word (after its data stores have been performed); nobody
// ever needs a read-modify-write, so one signal costs one store and one poll.
template <bool LOCAL = false>
__device__ __forceinline__ void flag_publish(unsigned long long *flag, unsigned long long epoch)
{
    if (LOCAL) __hip_atomic_store(flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    else __hip_atomic_store(flag, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Which die (XCC) of the device this wave runs on.
__device__ __forceinline__ uint32_t die_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)); }

// Flags of the die-local form carry the publisher's die in bits 57..60 (die + 1) above the epoch's low 57
// bits.  Like flags_wait_all; *same_die is set to whether every publisher's die is `die`.
constexpr unsigned long long kEpochMask57 = (1ull << 57) - 1;
__device__ __forceinline__ unsigned long long flag_with_die(unsigned long long epoch, uint32_t die) {
    return (epoch & kEpochMask57) | ((unsigned long long)(die + 1) << 57);
}
__device__ __forceinline__ bool flags_wait_all_local(const unsigned long long *flags, int n, unsigned long long epoch,
                                                     uint32_t spin_limit, int lane, uint32_t die, bool *same_die)
{
    const unsigned long long want = flag_with_die(epoch, die);
    for (uint32_t i = 0; i < spin_limit; ++i) {
        unsigned long long v = want;
        if (lane < n) v = __hip_atomic_load(flags + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__all((v & kEpochMask57) == (want & kEpochMask57))) {
            asm volatile("" ::: "memory");
            *same_die = __all(v == want);
            return true;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    *same_die = true;
    return false;
}

// Every lane of the calling wave polls until the first n (<= 64) words at
// `flags` all hold `epoch`; lane i watches word i.  At most `spin_limit` polls:
// returns false on timeout so that every wave still reaches the end of the
// kernel.  Loads issued after a true return observe everything the publishers
// stored coherently before publishing.
__device__ __forceinline__ bool flags_wait_all(const unsigned long long *flags, int n, unsigned long long epoch,
                                               uint32_t spin_limit, int lane)
{
    for (uint32_t i = 0; i < spin_limit; ++i) {
        unsigned long long v = epoch;
        if (lane < n) v = __hip_atomic_load(flags + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__all(v == epoch)) {
            asm volatile("" ::: "memory");
            return true;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    return false;
}

}  // namespace sv
