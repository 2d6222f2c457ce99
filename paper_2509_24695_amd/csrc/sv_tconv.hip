// C ABI of the temporal convolution (include/sv_tconv.h): argument checks and launches.
#include "../../include/sv_tconv.h"
#include "../../include/sv_measure.h"

#include <mutex>

#include "tconv_mfma.hpp"

namespace {

using namespace sv;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    const auto pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    return pa < pb + nb && pb < pa + na;
}

// The tile kernel needs its 128 KB of dynamic LDS allowed once per device.
bool tconv_kernel_ready()
{
    static bool ready[64] = {};
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (!ready[dev]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(tconv_mfma<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kTcLdsBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(tconv_mfma<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kTcLdsBytes) != hipSuccess)
            return false;
        ready[dev] = true;
    }
    return true;
}

// The tile kernel for a measurement variant (0 = the library's own), readied once per device.
using TconvKernel = void (*)(TconvArgs);
TconvKernel variant_kernel(int variant)
{
    switch (variant) {
    case 1: return tconv_mfma<false, 1>;
    case 2: return tconv_mfma<false, 2>;
    case 3: return tconv_mfma<false, 3>;
    default: return tconv_mfma<false, 0>;
    }
}
bool variant_kernel_ready(int variant)
{
    static bool ready[64][4] = {};
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (!ready[dev][variant]) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(variant_kernel(variant)),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kTcLdsBytes) != hipSuccess)
            return false;
        ready[dev][variant] = true;
    }
    return true;
}

sv_status tconv_enqueue(int variant, const void *x, const void *W, const void *cache_in, void *y, void *cache_out,
                        int32_t B, int32_t T, int32_t HW, int32_t D, int32_t dtype, void *stream)
{
    if (!x || !W || !y) return SV_ERR_NULL;
    if (B <= 0 || T <= 0 || HW <= 0 || D <= 0) return SV_ERR_SHAPE;
    if (dtype != SV_BF16) return SV_ERR_UNSUPPORTED;
    if (D % 8 != 0) return SV_ERR_UNSUPPORTED;
    const int64_t M = (int64_t)B * T * HW;
    if (M >= (int64_t)1 << 31 || (int64_t)3 * D * D >= (int64_t)1 << 31 || D > kTcMaxD) return SV_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(W) || !aligned16(y) || !aligned16(cache_in) || !aligned16(cache_out))
        return SV_ERR_ALIGN;
    const size_t tok_bytes = (size_t)M * D * 2, w_bytes = (size_t)3 * D * D * 2, cache_bytes = (size_t)B * HW * D * 2;
    if (overlaps(y, tok_bytes, x, tok_bytes) || overlaps(y, tok_bytes, W, w_bytes) ||
        (cache_in && overlaps(y, tok_bytes, cache_in, cache_bytes)))
        return SV_ERR_SHAPE;
    // the new cache is copied out of x after y is complete: it may replace cache_in, nothing else
    if (cache_out && (overlaps(cache_out, cache_bytes, y, tok_bytes) || overlaps(cache_out, cache_bytes, x, tok_bytes) ||
                      overlaps(cache_out, cache_bytes, W, w_bytes)))
        return SV_ERR_SHAPE;
    if (variant != 0 && D % kTcBK != 0) return SV_ERR_UNSUPPORTED;
    if (!(variant == 0 ? tconv_kernel_ready() : variant_kernel_ready(variant))) return SV_ERR_LAUNCH;

    TconvArgs a;
    a.x = static_cast<const uint16_t *>(x);
    a.W = static_cast<const uint16_t *>(W);
    a.cache = static_cast<const uint16_t *>(cache_in);
    a.y = static_cast<uint16_t *>(y);
    a.B = B; a.T = T; a.HW = HW; a.D = D;
    a.tiles_m = (int)((M + kTcBM - 1) / kTcBM);
    a.tiles_n = (D + kTcBN - 1) / kTcBN;
    const int64_t wgs = tc_grid_size((int64_t)a.tiles_m * a.tiles_n);
    if (wgs >= (int64_t)1 << 31) return SV_ERR_SHAPE;
    auto hs = static_cast<hipStream_t>(stream);
    if (variant != 0) variant_kernel(variant)<<<dim3((unsigned)wgs), kThreads, kTcLdsBytes, hs>>>(a);
    else if (D % kTcBK == 0) tconv_mfma<false><<<dim3((unsigned)wgs), kThreads, kTcLdsBytes, hs>>>(a);
    else tconv_mfma<true><<<dim3((unsigned)wgs), kThreads, kTcLdsBytes, hs>>>(a);
    if (hipGetLastError() != hipSuccess) return SV_ERR_LAUNCH;
    if (cache_out) {
        const int64_t vecs = (int64_t)B * HW * D / 8;
        const int blocks = (int)((vecs + kThreads - 1) / kThreads < 2048 ? (vecs + kThreads - 1) / kThreads : 2048);
        tconv_cache_store<<<blocks, kThreads, 0, hs>>>(a.x, static_cast<uint16_t *>(cache_out), B, T, HW, D);
        if (hipGetLastError() != hipSuccess) return SV_ERR_LAUNCH;
    }
    return SV_OK;
}

}  // namespace

extern "C" sv_status sv_tconv_block_step(const void *x, const void *W, const void *cache_in, void *y, void *cache_out,
                                         int32_t B, int32_t T, int32_t HW, int32_t D, int32_t dtype, void *stream)
{
    return tconv_enqueue(0, x, W, cache_in, y, cache_out, B, T, HW, D, dtype, stream);
}

extern "C" sv_status sv_measure_tconv_variant(int32_t variant, const void *x, const void *W, const void *cache_in, void *y,
                                              int32_t B, int32_t T, int32_t HW, int32_t D, void *stream)
{
    if (variant < 0 || variant > 3) return SV_ERR_RANGE;
    return tconv_enqueue(variant, x, W, cache_in, y, nullptr, B, T, HW, D, SV_BF16, stream);
}
