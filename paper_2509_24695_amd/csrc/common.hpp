// Shared device-side helpers for the gfx950 linear-attention kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tile_walk.hpp"

namespace sv {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kThreads = 256;        // every kernel here runs 4 waves per workgroup
constexpr int kWavesPerWg = kThreads / kWave;
constexpr int kMaxChunks = 32;       // upper bound on token chunks per head (workspace sizing)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Element strides of a [B][H][N][d] token tensor (d contiguous).
struct TokStrides {
    int64_t b, h, n;
};

// ---- bf16 <-> fp32 on raw bit patterns -------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Round to nearest even (hardware conversion on gfx950).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
    return __builtin_bit_cast(uint16_t, (__bf16)x);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// ReLU feature map on two packed bf16 values: a negative bf16 is a negative
// int16, so a signed 16-bit max with zero clears it (and turns -0 into +0).
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t w) {
    const s16x2 zero = {0, 0};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, w), zero));
}
__device__ __forceinline__ u32x4 relu_bf16x8(u32x4 v) {
    v.x = relu_bf16x2(v.x); v.y = relu_bf16x2(v.y); v.z = relu_bf16x2(v.z); v.w = relu_bf16x2(v.w);
    return v;
}

// ---- RoPE after ReLU (numerator of the Sec. 3.2 equation) ----------------------------------------
// A rotation table row holds d/2 (cos, sin) fp32 pairs of one token; feature pair
// (2p, 2p+1) is turned by angle p:  y[2p] = x[2p] cos - x[2p+1] sin,  y[2p+1] = x[2p] sin + x[2p+1] cos.
// A 32-bit word of a bf16 token row is exactly one such pair.
__device__ __forceinline__ uint32_t rope_rotate_pair(uint32_t w, float c, float s) {
    const float a = bf16_lo(w), b = bf16_hi(w);
    return pack_bf16x2(a * c - b * s, a * s + b * c);
}
// Four pairs (16 bytes of a token row) with their four (cos, sin) entries.
__device__ __forceinline__ u32x4 rope_rotate_bf16x8(u32x4 w, f32x4 cs01, f32x4 cs23) {
    u32x4 r;
    r.x = rope_rotate_pair(w.x, cs01.x, cs01.y);
    r.y = rope_rotate_pair(w.y, cs01.z, cs01.w);
    r.z = rope_rotate_pair(w.z, cs23.x, cs23.y);
    r.w = rope_rotate_pair(w.w, cs23.z, cs23.w);
    return r;
}
// ---- range-checked streaming access ------------------------------------------------------------
//
// Token tiles are addressed through buffer resources: the hardware compares each
// lane's byte offset with the resource's size, returns zeros for loads at or past
// it and drops such stores.  Ragged tails and tiles past the end of a wave's share
// therefore need no branch, every stage of a software pipeline issues the same
// number of memory instructions, and the compiler can wait for exactly the
// loads it needs (s_waitcnt vmcnt(n)) while later ones stay in flight.  Offsets are
// 32-bit: the host routes tensors whose heads span 2 GiB or more to other kernels.
using rsrc_t = __amdgpu_buffer_rsrc_t;

// `p` must be wave-uniform.  Bytes [0, bytes) are addressable.
__device__ __forceinline__ rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

// Tokens are read once and outputs written once, so with SV_STREAM_NT both are
// marked non-temporal.
#ifndef SV_STREAM_NT
#define SV_STREAM_NT 1
#endif
#ifndef SV_STORE_NT
#define SV_STORE_NT SV_STREAM_NT
#endif
__device__ __forceinline__ u32x4 load_stream16(rsrc_t r, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, SV_STREAM_NT ? 2 : 0);
}
// Token bytes that one wave reads (STREAM) or that a second wave reads again soon after.
template <bool STREAM> __device__ __forceinline__ u32x4 load_tokens16(rsrc_t r, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, STREAM && SV_STREAM_NT ? 2 : 0);
}
__device__ __forceinline__ void store_stream16(rsrc_t r, uint32_t off, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, SV_STORE_NT ? 2 : 0);
}
// Cached 16-byte load (rotation table: shared by all heads, worth keeping in L2).
__device__ __forceinline__ f32x4 load_cached16(rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
}

// ---- typed scalar access used by the generic (any dtype) kernels --------------------------

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float x) { *p = x; }
};
template <> struct Elem<uint16_t> {   // bf16 bit patterns
    static __device__ __forceinline__ float load(const uint16_t *p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t *p, float x) { *p = f32_to_bf16_bits(x); }
};

// Tiles of a token range are dealt to chunks as evenly as integers allow:
// chunk c of C owns tiles [c*T/C, (c+1)*T/C).
__host__ __device__ __forceinline__ int chunk_tile_begin(int c, int C, int T) {
    return (int)(((int64_t)c * T) / C);
}

// Orders this wave's LDS traffic for the compiler; the hardware already executes
// one wave's LDS instructions in issue order, so no s_barrier is involved.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier for handing LDS over between waves.  __syncthreads() alone does not do: the compiler
// has been seen to move LDS reads that stand before it to behind it (two barriers in a row, the reads
// after both), where another wave, already past the barrier, may have overwritten the memory.  The
// assembly statement is opaque to the compiler (no memory operation crosses it in either direction) and
// waits for this wave's LDS traffic, reads included, before the waves meet; the fences keep the meaning
// that __syncthreads() has for global memory.
__device__ __forceinline__ void wg_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// All LDS traffic of this wave is done, then all waves of the workgroup meet.
// Global memory traffic is not waited for.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace sv
