// Streaming yardsticks (include/sv_measure.h): a pure read and a pure copy with the access width
// of the attention kernels (16 bytes per lane).
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
