// Yardsticks (include/sv_measure.h): a pure read and a pure copy with the access width of the
// attention kernels (16 bytes per lane), and a pure matrix-core instruction stream with the shape
// of the temporal convolution's inner loop.
#include "../../include/sv_measure.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256, kUnroll = 8;

// Workgroup g owns vectors [g * per_wg, (g + 1) * per_wg) of the n_vec 16-byte vectors.
__global__ __launch_bounds__(kThreads) void stream_read(const u32x4 *__restrict__ src, size_t n_vec, u32x4 *sink)
{
    const size_t per_wg = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = per_wg * blockIdx.x, hi = lo + per_wg < n_vec ? lo + per_wg : n_vec;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = lo + threadIdx.x;
    for (; i + (kUnroll - 1) * kThreads < hi; i += kUnroll * kThreads) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u];
    }
    for (; i < hi; i += kThreads) acc ^= __builtin_nontemporal_load(src + i);
    if (acc.x == 0x12345678u && acc.y == 77u) *sink = acc;
}

__global__ __launch_bounds__(kThreads) void stream_copy(const u32x4 *__restrict__ src, size_t n_vec, u32x4 *__restrict__ dst)
{
    const size_t per_wg = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t lo = per_wg * blockIdx.x, hi = lo + per_wg < n_vec ? lo + per_wg : n_vec;
    size_t i = lo + threadIdx.x;
    for (; i + (kUnroll - 1) * kThreads < hi; i += kUnroll * kThreads) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) __builtin_nontemporal_store(v[u], dst + i + u * kThreads);
    }
    for (; i < hi; i += kThreads) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// What one workgroup of the temporal convolution issues per K-step of 32, and nothing else: four waves, each
// 2 x 16 MFMAs (32x32x16 bf16) on a 4 x 4 grid of accumulators, operands held in registers (two sets taken in
// turn, as the convolution alternates its two operand buffers).  No LDS, no memory traffic, no barrier.
typedef __attribute__((ext_vector_type(8))) __bf16 ys_bf16x8;
typedef __attribute__((ext_vector_type(16))) float ys_f32x16;

__global__ __launch_bounds__(kThreads) void mfma_stream(int steps, float *sink)
{
    // operand bits that differ per lane, register and set: +-[1, 2) with mixed mantissas
    union { ys_bf16x8 v; uint16_t h[8]; } op[2][8];
    uint32_t x = (threadIdx.x + 1u) * 2654435761u ^ (blockIdx.x * 40503u);
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x = x * 1664525u + 1013904223u;
                op[kk][m].h[e] = (uint16_t)(0x3F80u | ((x >> 16) & 0x807Fu));
            }
    ys_f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    for (int s = 0; s < steps; ++s) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int m = 0; m < 16; ++m)
                acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[kk][m >> 2].v, op[kk][4 + (m & 3)].v,
                                                                              acc[m >> 2][m & 3], 0, 0, 0);
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) t += acc[i][j][r];
    if (t == 12345.678f) *sink = t;      // keeps the products alive; practically never true
}

}  // namespace sv

namespace {

using namespace sv;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

sv_status check(const void *a, const void *b, size_t bytes, int32_t wgs)
{
    if (!a || !b) return SV_ERR_NULL;
    if (!aligned16(a) || !aligned16(b) || bytes % 16 != 0) return SV_ERR_ALIGN;
    if (wgs < 1 || wgs > (1 << 20)) return SV_ERR_SHAPE;
    return SV_OK;
}

}  // namespace

extern "C" sv_status sv_stream_read(const void *src, size_t bytes, void *sink, int32_t wgs, void *stream)
{
    const sv_status st = check(src, sink, bytes, wgs);
    if (st != SV_OK) return st;
    if (bytes == 0) return SV_OK;
    stream_read<<<dim3((unsigned)wgs), kThreads, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const u32x4 *>(src), bytes / 16, static_cast<u32x4 *>(sink));
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH;
}

extern "C" sv_status sv_stream_copy(const void *src, void *dst, size_t bytes, int32_t wgs, void *stream)
{
    const sv_status st = check(src, dst, bytes, wgs);
    if (st != SV_OK) return st;
    const auto ps = reinterpret_cast<uintptr_t>(src), pd = reinterpret_cast<uintptr_t>(dst);
    if (ps < pd + bytes && pd < ps + bytes) return SV_ERR_SHAPE;
    if (bytes == 0) return SV_OK;
    stream_copy<<<dim3((unsigned)wgs), kThreads, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<const u32x4 *>(src), bytes / 16, static_cast<u32x4 *>(dst));
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH;
}

extern "C" sv_status sv_mfma_stream(int32_t wgs, int32_t steps, void *sink, void *stream)
{
    if (!sink) return SV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(sink) & 3u) != 0) return SV_ERR_ALIGN;
    if (wgs < 1 || wgs > (1 << 20) || steps < 0 || steps > (1 << 20)) return SV_ERR_SHAPE;
    if (steps == 0) return SV_OK;
    mfma_stream<<<dim3((unsigned)wgs), kThreads, 0, static_cast<hipStream_t>(stream)>>>(steps, static_cast<float *>(sink));
    return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH;
}
