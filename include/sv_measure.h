/*
 * sv_measure.h - yardsticks (MI355X, gfx950; part of libsvlinattn.so).
 *
 * Not part of the method of the paper: two kernels that do nothing but move
 * bytes, for callers that want to know what this device gives a pure stream of
 * a given size - the ceiling the attention kernels (all of them bound by memory
 * traffic) are measured against beside the published peak - and one that does
 * nothing but issue matrix-core instructions (sv_mfma_stream, below).
 *
 * The two streaming calls take device pointers, work on `stream` (hipStream_t passed as void*,
 * NULL = default stream), return after enqueueing, allocate nothing and keep
 * nothing.  `wgs` workgroups of 256 threads each walk a contiguous share of the
 * buffer with 16-byte accesses, eight in flight per thread.
 *
 * Errors (checked on the host before any launch): SV_ERR_NULL for a null
 * pointer, SV_ERR_ALIGN if a pointer or `bytes` is not a multiple of 16,
 * SV_ERR_SHAPE if wgs is outside [1, 1048576] or (copy) the buffers overlap,
 * SV_ERR_LAUNCH if the launch failed.  bytes == 0 is legal and launches nothing.
 */
#ifndef SV_MEASURE_H
#define SV_MEASURE_H

#include "sv_linattn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Reads src[0, bytes) once.  `sink` is 16 bytes of device memory that the kernel
 * may write (it does so only for one bit pattern of the data in a million; the
 * store is what keeps the loads alive). */
sv_status sv_stream_read(const void *src, size_t bytes, void *sink, int32_t wgs, void *stream);

/* dst[0, bytes) = src[0, bytes). */
sv_status sv_stream_copy(const void *src, void *dst, size_t bytes, int32_t wgs, void *stream);

/* The matrix-core instruction stream of the temporal convolution (sv_tconv.h) with everything else taken
 * away: `wgs` workgroups of four waves, each wave issuing 32 * steps v_mfma_f32_32x32x16_bf16 on a 4 x 4 grid
 * of accumulators from operands that stay in registers (one 256 x 256 output tile of the convolution is
 * steps = 3 * D / 32; a workgroup does steps * 4 194 304 flop).  What this device gives that stream at a given
 * number of busy compute units is the ceiling of any kernel built on it.  `sink` is 4 bytes of device memory,
 * 4-byte aligned, that the kernel may write (for one value of its sums; the store keeps the products alive).
 * Enqueues on `stream` and returns; allocates nothing.  SV_ERR_NULL / SV_ERR_ALIGN for sink, SV_ERR_SHAPE if
 * wgs is outside [1, 1048576] or steps outside [0, 1048576]; steps == 0 launches nothing. */
sv_status sv_mfma_stream(int32_t wgs, int32_t steps, void *sink, void *stream);

/* sv_linattn_apply for bf16 tokens and d = 64 in four forms of its kernel, for A/B measurements of two
 * design choices (same arguments, checks, launch shape and results to rounding as sv_linattn_apply; no
 * passage of the paper of its own):
 *   variant 0  the kernel sv_linattn_apply launches: the head's state S lives in each wave's registers as
 *              matrix-core operands for the whole token range, and the denominators phi(Q_i).z come out of
 *              the same matrix-core pass (z as two extra operand rows, one cross-lane exchange);
 *   variant 1  S kept in LDS instead (one copy per workgroup) and read again for every 32-token tile,
 *              denominators as in variant 0;
 *   variant 2  S in registers, denominators on the vector ALU: per lane 32 multiply-adds against the key
 *              sums, then the two half-waves exchange their partial sums (a wavefront-level reduction);
 *   variant 3  S in LDS and denominators on the vector ALU.
 * SV_ERR_RANGE for another variant, SV_ERR_UNSUPPORTED unless the descriptor is SV_BF16 with d = 64 and
 * heads below 2 GiB.  The first call of a variant on a device sets a kernel attribute: not under graph
 * capture. */
sv_status sv_measure_apply_variant(int32_t variant, const void *Q, const sv_tensor_desc *q,
                                   int32_t tok_begin, int32_t tok_end,
                                   const float *S, const float *z, float eps, void *O, void *stream);

/* The tile kernel of sv_tconv_block_step (sv_tconv.h; same arguments without cache_out and dtype, same checks,
 * same grid, bf16 only) with parts of its loop left out, to time what each part costs (no passage of the paper):
 *   variant 0  the kernel sv_tconv_block_step launches;
 *   variant 1  without the loads from memory into LDS inside the tile loop (the prologue's stay);
 *   variant 2  without the operand reads from LDS inside the tile loop;
 *   variant 3  without both: the matrix-core instructions, the barriers, prologue and epilogue.
 * Variants 1-3 read the same memory and write every element of y, but what they write is not the convolution
 * (finite values for finite inputs).  SV_ERR_RANGE for another variant, SV_ERR_UNSUPPORTED for variants 1-3
 * unless D is a multiple of 32; otherwise the errors of sv_tconv_block_step.  The first call of a variant on a
 * device sets a kernel attribute: not under graph capture. */
sv_status sv_measure_tconv_variant(int32_t variant, const void *x, const void *W, const void *cache_in, void *y,
                                   int32_t B, int32_t T, int32_t HW, int32_t D, void *stream);

/* For tests of a safety net, no passage of the paper.  On the 8-die part the one-launch block step places all
 * workgroups of a head on one die (workgroup ids go round the dies) and lets them exchange their partial states
 * through that die's L2; every workgroup publishes the die it really runs on, and a head found on more than one
 * die stores nothing and sets the workspace's timeout mark (sv_linattn_workspace_status).  This call makes all
 * later block steps of the process place heads as if the device had `dies` dies (1, 2 or 4: heads then do end up
 * on several dies, so every such step must give up and report; any other value restores the real count).  The
 * kernels run to their end either way. */
void sv_measure_assume_dies(int32_t dies);

#ifdef __cplusplus
}
#endif

#endif /* SV_MEASURE_H */
