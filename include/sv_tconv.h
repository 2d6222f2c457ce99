/*
 * sv_tconv.h - C ABI of the block-causal temporal convolution of the Mix-FFN
 * (MI355X, gfx950; part of libsvlinattn.so).
 *
 * The Mix-FFN of the SANA-Video paper (arXiv 2509.24695, Sec. 3.2, "Mix-FFN with
 * Spatial-Temporal Mixture") ends in a 1-D convolution along the frame axis
 * with a shortcut connection; Sec. 3.3.1 ("Block Causal Mix-FFN") makes it
 * causal over blocks: the frame in front of a block is the cached last frame
 * of the previous block, the frame behind it is all zeros, the kernel size is
 * 3.  With x the block's input, frames t = 0..T-1, positions p, channels o:
 *
 *     y[b][t][p][o] = x[b][t][p][o]
 *                   + sum_i W[0][o][i] * x[b][t-1][p][i]     (t = 0: cache_in[b][p][i], or 0)
 *                   + sum_i W[1][o][i] * x[b][t  ][p][i]
 *                   + sum_i W[2][o][i] * x[b][t+1][p][i]     (t = T-1: 0)
 *     cache_out[b][p][:] = x[b][T-1][p][:]
 *
 * The paper gives neither the channel structure nor the tap order; this
 * library takes the convolution as dense over channels, without bias, taps
 * applied as a cross-correlation, and caches the module's input frame.  A call
 * without cache over the whole clip is the convolution of the bidirectional
 * model (zero padding on both sides).
 */
#ifndef SV_TCONV_H
#define SV_TCONV_H

#include "sv_linattn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* One block through the temporal convolution with shortcut.
 *
 *  x          device, [B][T][HW][D] dense, D contiguous              (read)
 *  W          device, [3][D][D] dense: W[tap][out][in]               (read)
 *  cache_in   device, [B][HW][D] dense, or NULL = empty cache (the state Alg. 1
 *             starts from): the frame in front of the block          (read)
 *  y          device, [B][T][HW][D] dense                            (written)
 *  cache_out  device, [B][HW][D] dense, or NULL: receives the block's last input
 *             frame.  NULL leaves the cache as it is, which is what every
 *             denoising step but the last wants (Alg. 1 replaces the conv cache
 *             once per block).  May be the same buffer as cache_in: it is written
 *             after y is complete.                                    (written)
 *  dtype      SV_BF16 only: bf16 storage, bf16 MFMA products accumulated in fp32
 *             over all 3*D terms, the shortcut added in fp32, one rounding to
 *             bf16 (nearest even).  SV_F32 returns SV_ERR_UNSUPPORTED.
 *
 * B, T, HW >= 1; D >= 8 and a multiple of 8; B*T*HW and 3*D*D below 2^31.  All
 * pointers 16-byte aligned.  y must not overlap x, W or cache_in; cache_out must not
 * overlap x, W or y (SV_ERR_SHAPE).  Inputs must
 * be finite.  Arguments are checked on the host before anything is launched; an
 * error other than SV_ERR_LAUNCH means nothing was written.  Work is enqueued
 * on `stream` (hipStream_t as void*, NULL = default stream); the library
 * allocates nothing and keeps no pointer.  Results are bit-reproducible (fixed
 * summation order, no atomics).  The first call on a device raises the kernel's
 * LDS limit (a function attribute): make it before capturing the stream into a
 * HIP graph; later calls only enqueue two kernels and may be captured. */
sv_status sv_tconv_block_step(const void *x, const void *W, const void *cache_in,
                              void *y, void *cache_out,
                              int32_t B, int32_t T, int32_t HW, int32_t D,
                              int32_t dtype, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SV_TCONV_H */
