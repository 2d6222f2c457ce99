// Shared device-side helpers for the gfx950 linear-attention kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
// Table entries for the 16-byte chunks a lane holds of a d = 64 tile in the coalesced layout
// (token tok0 + lane/8 + 8i, pairs 4*(lane%8) .. +3).  Rows past t1 are not touched.
template <int TILE>
__device__ __forceinline__ void rope_tile_load(const float *__restrict__ rope, int tok0, int t1, int lane,
                                               f32x4 (&cs)[TILE / 8][2])
{
#pragma unroll
    for (int i = 0; i < TILE / 8; ++i) {
        const int tok = tok0 + (lane >> 3) + 8 * i;
        f32x4 a = {1.f, 0.f, 1.f, 0.f}, b = {1.f, 0.f, 1.f, 0.f};
        if (tok < t1) {
            const float *row = rope + (int64_t)tok * 64 + (lane & 7) * 8;
            a = *reinterpret_cast<const f32x4 *>(row);
            b = *reinterpret_cast<const f32x4 *>(row + 4);
        }
        cs[i][0] = a;
        cs[i][1] = b;
    }
}

// Streaming 16-byte global accesses.  Tokens are read once and outputs written
// once, so with SV_STREAM_NT both are marked non-temporal.
#ifndef SV_STREAM_NT
#define SV_STREAM_NT 1
#endif
__device__ __forceinline__ u32x4 load_stream16(const void *p) {
#if SV_STREAM_NT
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
#else
    return *reinterpret_cast<const u32x4 *>(p);
#endif
}
#ifndef SV_STORE_NT
#define SV_STORE_NT SV_STREAM_NT
#endif
__device__ __forceinline__ void store_stream16(void *p, u32x4 v) {
#if SV_STORE_NT
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
#else
    *reinterpret_cast<u32x4 *>(p) = v;
#endif
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

}  // namespace sv
