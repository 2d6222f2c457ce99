// Block-causal temporal convolution of the Mix-FFN with shortcut (Sec. 3.3.1, "Block Causal
// Mix-FFN"; Mix-FFN paragraph of Sec. 3.2) as one implicit GEMM on the matrix cores.
//
//   y[g][o] = x[g][o] + sum_tap sum_i W[tap][o][i] * src_tap(g)[i]
//
// for token rows g = (b, t, p) of a block of T frames x HW positions, where src_tap(g) is the row
// of the same position in frame t + tap - 1: a row of x, the cached last frame of the previous
// block for frame -1 (zeros without a cache), zeros for frame T.  So the A operand of the GEMM
// is x read three times with its rows shifted by -HW, 0, +HW tokens, the contraction runs over
// 3*D, and nothing is materialised.  Rows that are zero (frame -1 without a cache, frame T,
// token and channel tails, the K tail when D is not a multiple of the K-step) are read from a
// row of zeros in device memory, so the loader has no special cases.
//
// Tiling: a workgroup of four waves (one per SIMD) owns a 256-token x 256-channel tile of y; wave
// (wm, wn) owns a 128 x 128 quadrant as 4 x 4 accumulators of v_mfma_f32_32x32x16_bf16.  Both
// operands are K-contiguous ([token][channel] and [out][in]), so a K-step of 32 is a [256][32]
// bf16 tile of each (16 KB + 16 KB), and LDS holds a ring of four such stages.
//
// Pipeline: operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: a
// wave's 64 lanes fill 1 KB of consecutive LDS, no staging registers, completion counted by
// vmcnt).  With one wave per SIMD nothing but the wave itself can fill the time the matrix core
// works, so every memory instruction sits between two MFMAs.  Step s (stage s & 3):
//   first half   16 MFMAs on operand registers of K-chunk 0; reads K-chunk 1 of stage s;
//                requests the B rows of step s+3
//   barrier      after waiting for this wave's loads of step s+1 and its own LDS reads
//   second half  16 MFMAs on K-chunk 1; reads K-chunk 0 of stage s+1; requests the A rows of
//                step s+4 into stage s (every wave has read it: the barrier has passed)
// so a tile is requested two to three steps before its first use.  Steps past the end
// repeat the last one into stages nobody reads: the loop body has no conditions.
//
// LDS rows are 64 bytes; the 16-byte chunk c of row r sits at chunk slot c ^ f(r),
// f(r) = ((r>>1)&3) ^ ((r>>3)&1), which spreads the 16-byte reads of consecutive rows (one matrix
// operand: 32 rows, one chunk column) over all banks whether the hardware serves 8 or 16 lanes
// per cycle; the lane that fills slot (r, c') therefore loads chunk c' ^ f(r) of row r.
#pragma once

#include "common.hpp"
#include "tconv_tiles.hpp"

namespace sv {

constexpr int kTcBM = 256, kTcBN = 256, kTcBK = 32;
constexpr int kTcTileBytes = kTcBM * kTcBK * 2;               // one operand tile of one K-step
constexpr int kTcStageBytes = 2 * kTcTileBytes;               // A and B
constexpr int kTcStages = 4;
constexpr int kTcLdsBytes = kTcStages * kTcStageBytes;
constexpr int kTcEpiPitch = 128 * 4 + 32;                     // fp32 row of a wave's quadrant in the epilogue
constexpr int kTcMaxD = 32768;                                // length of the row of zeros
static_assert(4 * 32 * kTcEpiPitch <= kTcLdsBytes, "epilogue staging fits in the operand ring");

// A row of zeros for operand rows that do not exist.  Never written.
static __device__ __align__(16) uint16_t tc_zero_row[kTcMaxD];

struct TconvArgs {
    const uint16_t *x, *W, *cache;     // cache may be null
    uint16_t *y;
    int B, T, HW, D;
    int tiles_m, tiles_n;              // token tiles, channel tiles
};

__device__ __forceinline__ uint32_t tc_swizzle(int r) { return (uint32_t)(((r >> 1) & 3) ^ ((r >> 3) & 1)); }

// 16 bytes per lane from global memory to LDS: lane l of the wave writes lds_wave_base + 16 l.
__device__ __forceinline__ void tc_load_to_lds(const uint16_t *src, unsigned char *lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// KTAIL: D is not a multiple of the K-step, the last K-step of a tap has chunks past the row end.
// SKIP: measurement variants (sv_measure_tconv_variant; the library's own calls use 0): bit 0 leaves the
// loads into LDS out of the tile loop, bit 1 the operand reads from LDS.  Such a launch touches the same
// memory and writes every element of y, but what it writes is not the convolution.
template <bool KTAIL, int SKIP = 0>
__global__ __launch_bounds__(kThreads) void tconv_mfma(TconvArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    int tm, tn;
    if (!tc_tile_of(a.tiles_m, a.tiles_n, (int)blockIdx.x, tm, tn)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int M = a.B * a.T * a.HW, D = a.D;
    const int m0 = tm * kTcBM, n0 = tn * kTcBN;
    const int KC = (D + kTcBK - 1) / kTcBK, steps = 3 * KC;

    // ---- loader role: one 16-byte chunk of rows r0 + 64 i of both operand tiles ------------------
    const int r0 = tid >> 2, c4 = (tid & 3) ^ (int)tc_swizzle(r0);   // c4: the chunk whose slot is this lane's
    int row_t[4], row_c[4];            // frame of the row (or a large value past M), cache row index
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g = m0 + r0 + 64 * i, gc = g < M ? g : M - 1;
        const int thw = a.T * a.HW, b = gc / thw, rem = gc - b * thw, t = rem / a.HW;
        row_t[i] = g < M ? t : 1 << 20;      // rows past the last token: every tap sees them as past the block
        row_c[i] = b * a.HW + (rem - t * a.HW);
    }
    const uint16_t *srcA[4], *srcB[4]; // the lane's chunk of each row at K-step 0 of the current tap
    auto set_tap = [&](int tap) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ts = row_t[i] + tap - 1;
            const bool front = ts < 0, zero = ts >= a.T || (front && !a.cache);
            const uint16_t *in_x = a.x + ((int64_t)(m0 + r0 + 64 * i) + (int64_t)(tap - 1) * a.HW) * D;
            const uint16_t *in_c = a.cache + (int64_t)row_c[i] * D;
            srcA[i] = (zero ? tc_zero_row : (front ? in_c : in_x)) + c4 * 8;
            const int n = n0 + r0 + 64 * i;
            srcB[i] = (n >= D ? tc_zero_row : a.W + ((int64_t)tap * D + n) * D) + c4 * 8;
        }
    };
    int tap_n = 0, kc_n = 0;           // the step to request next
    auto advance = [&]() {
        if (kc_n + 1 < KC) {
            ++kc_n;
        } else if (tap_n < 2) {
            kc_n = 0;
            set_tap(++tap_n);
        }                              // else: stay on the last step
    };
    // Source of load m (m < 4: A row pass m, else B row pass m - 4) of the step to request next.
    auto source = [&](int m) -> const uint16_t * {
        const uint16_t *p = (m < 4 ? srcA[m] : srcB[m - 4]) + kc_n * kTcBK;
        if (KTAIL && kc_n * kTcBK + c4 * 8 >= D) p = tc_zero_row;
        return p;
    };
    auto request_one = [&](int stage, int m) {
        unsigned char *dst = lds + stage * kTcStageBytes + (m < 4 ? 0 : kTcTileBytes) + ((m & 3) * 64 + wave * 16) * 64;
        tc_load_to_lds(source(m), dst);
    };

    // ---- consumer role ------------------------------------------------------------------------------
    uint32_t ko[2];                    // byte offset of K-chunk pair kk inside the lane's operand row
    {
        const uint32_t g = (uint32_t)(lane >> 5) ^ tc_swizzle(lane & 31);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) ko[kk] = (((uint32_t)kk << 1) ^ g) << 4;
    }
    const uint32_t rdA = (uint32_t)(wm * 128 + (lane & 31)) * 64u;
    const uint32_t rdB = (uint32_t)kTcTileBytes + (uint32_t)(wn * 128 + (lane & 31)) * 64u;
    // operand m of a set: A row block m (m < 4) or B row block m - 4
    auto operand = [&](int stage, int kk, int m) -> bf16x8 {
        const unsigned char *base = lds + stage * kTcStageBytes + (m < 4 ? rdA : rdB) + (m & 3) * 2048 + ko[kk];
        return *reinterpret_cast<const bf16x8 *>(base);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    bf16x8 op[2][8];                   // op[kk][0..3] = A row blocks, op[kk][4..7] = B row blocks

    // ---- prologue: steps 0..2 and the A half of step 3 requested, step 0 arrived --------------------
    set_tap(0);
#pragma unroll
    for (int st = 0; st < kTcStages - 1; ++st) {
#pragma unroll
        for (int m = 0; m < 8; ++m) request_one(st, m);
        advance();
    }
#pragma unroll
    for (int m = 0; m < 4; ++m) request_one(kTcStages - 1, m);
    if (SKIP & 1) {                    // no loads in the loop: the ring is filled here, once, and read over and over
#pragma unroll
        for (int m = 4; m < 8; ++m) request_one(kTcStages - 1, m);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(20)\n\ts_barrier" ::: "memory");
#pragma unroll
    for (int m = 0; m < 8; ++m) op[0][m] = operand(0, 0, m);
    if (SKIP & 2) {
#pragma unroll
        for (int m = 0; m < 8; ++m) op[1][m] = operand(0, 1, m);
    }

    // A load instruction keeps the wave from issuing for longer than one MFMA runs, so the eight
    // loads of a step are spread out: one after every second MFMA of the second half of one step
    // (A rows) and of the first half of the next (B rows).
    for (int s = 0; s < steps; ++s) {
        const int cur = s & 3, nxt = (s + 1) & 3, prv = (s + 3) & 3;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[0][m >> 2], op[0][4 + (m & 3)],
                                                                          acc[m >> 2][m & 3], 0, 0, 0);
            if (!(SKIP & 2) && m < 8) op[1][m] = operand(cur, 1, m);
            if (!(SKIP & 1) && m >= 8 && (m & 1)) request_one(prv, 4 + ((m - 8) >> 1));     // B rows of step s+3
            __builtin_amdgcn_sched_barrier(0);
        }
        advance();
        // this wave's loads of step s+1 have landed (those of steps s+2 and s+3 may be in flight) and its reads
        // of stage s are done; then so have everybody's
        asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[1][m >> 2], op[1][4 + (m & 3)],
                                                                          acc[m >> 2][m & 3], 0, 0, 0);
            if (!(SKIP & 2) && m < 8) op[0][m] = operand(nxt, 0, m);
            if (!(SKIP & 1) && m >= 8 && (m & 1)) request_one(cur, (m - 8) >> 1);           // A rows of step s+4
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // ---- epilogue: y = bf16(x + acc), 32 token rows of the wave's quadrant at a time through LDS ----
    // (nobody reads the operand ring any more; each wave uses its own region).  The shortcut's x rows
    // are requested one 32-row group ahead, so their latency is paid once per tile, not once per row.
    unsigned char *epi = lds + wave * (32 * kTcEpiPitch);
    const int er = lane >> 4, ec = lane & 15;                 // reader: row in a group of four, 8-channel chunk
    const int n = n0 + wn * 128 + ec * 8;
    const bool col_ok = n < D;
    const int n_ld = col_ok ? n : 0;                          // lanes past the last channel load a valid address
    u32x4 xin[2][8];
    auto load_x = [&](int buf, int i) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int64_t g = (int64_t)m0 + wm * 128 + i * 32 + it * 4 + er;
            xin[buf][it] = *reinterpret_cast<const u32x4 *>(a.x + (g < M ? g : (int64_t)M - 1) * D + n_ld);
        }
    };
    load_x(0, 0);
    // the repeated loads of the last steps must not land on the epilogue's staging
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i + 1 < 4) load_x((i + 1) & 1, i + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), col = j * 32 + (lane & 31);
                *reinterpret_cast<float *>(epi + row * kTcEpiPitch + col * 4) = acc[i][j][r];
            }
        wave_lds_fence();
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int row = it * 4 + er;
            const int64_t g = (int64_t)m0 + wm * 128 + i * 32 + row;
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(epi + row * kTcEpiPitch + ec * 32);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(epi + row * kTcEpiPitch + ec * 32 + 16);
            if (g < M && col_ok) {
                const u32x4 x4 = xin[i & 1][it];
                u32x4 out;
                out.x = pack_bf16x2(bf16_lo(x4.x) + lo.x, bf16_hi(x4.x) + lo.y);
                out.y = pack_bf16x2(bf16_lo(x4.y) + lo.z, bf16_hi(x4.y) + lo.w);
                out.z = pack_bf16x2(bf16_lo(x4.z) + hi.x, bf16_hi(x4.z) + hi.y);
                out.w = pack_bf16x2(bf16_lo(x4.w) + hi.z, bf16_hi(x4.w) + hi.w);
                *reinterpret_cast<u32x4 *>(a.y + g * D + n) = out;
            }
        }
        wave_lds_fence();
    }
}

// New cache = last input frame of the block: cache[b][p][:] = x[b][T-1][p][:], 16 bytes per thread.
__global__ __launch_bounds__(kThreads) void tconv_cache_store(const uint16_t *x, uint16_t *cache, int B, int T, int HW, int D)
{
    const int64_t per_batch = (int64_t)HW * D / 8, total = per_batch * B;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = e / per_batch, r = e - b * per_batch;
        const u32x4 v = reinterpret_cast<const u32x4 *>(x + ((b * T + (T - 1)) * (int64_t)HW) * D)[r];
        reinterpret_cast<u32x4 *>(cache + b * (int64_t)HW * D)[r] = v;
    }
}

}  // namespace sv
