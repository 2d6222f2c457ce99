// Block-causal temporal convolution of the Mix-FFN with shortcut (Sec. 3.3.1, "Block Causal
// Mix-FFN"; Mix-FFN paragraph of Sec. 3.2) as one implicit GEMM on the matrix cores.
//
//   y[g][o] = x[g][o] + sum_tap sum_i W[tap][o][i] * src_tap(g)[i]
//
// for token rows g = (b, t, p) of a block of T frames x HW positions, where src_tap(g) is the row
// of the same position in frame t + tap - 1: a row of x, the cached last frame of the previous
// block for frame -1 (zeros without a cache), zeros for frame T.  So the A operand of the GEMM
// is x read three times with its rows shifted by -HW, 0, +HW tokens, the contraction runs over
// 3*D, and nothing is materialised.
//
// Tiling: a workgroup of four waves owns a 256-token x 256-channel tile of y; wave (wm, wn) owns
// a 128 x 128 quadrant as 4 x 4 accumulators of v_mfma_f32_32x32x16_bf16.  Both operands are
// K-contiguous ([token][channel] and [out][in]), so a K-step of 64 is a [256][64] bf16 tile of
// each (32 KB + 32 KB), double-buffered in LDS: global loads of step s+1 are issued before the
// products of step s and land in registers meanwhile, then go to the other LDS buffer, one
// barrier per step.  LDS rows are 128 bytes; the 16-byte chunk c of row r sits at chunk slot
// c ^ f(r), f(r) = 4*(r&1) ^ ((r>>1)&7), which spreads the 16-byte reads of consecutive rows
// (one matrix operand: 32 rows, one chunk column) over all banks and keeps the writes of a
// wave (8 rows x 8 chunks) contiguous.
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kTcBM = 256, kTcBN = 256, kTcBK = 64;
constexpr int kTcTileBytes = kTcBM * kTcBK * 2;               // one operand tile of one K-step
constexpr int kTcStageBytes = 2 * kTcTileBytes;               // A and B
constexpr int kTcLdsBytes = 2 * kTcStageBytes;                // double-buffered
constexpr int kTcGroupM = 4;                                  // token tiles per XCD group
constexpr int kTcEpiPitch = 128 * 4 + 32;                     // fp32 row of a wave's quadrant in the epilogue

struct TconvArgs {
    const uint16_t *x, *W, *cache;     // cache may be null
    uint16_t *y;
    int B, T, HW, D;
    int tiles_m, tiles_n, groups;      // token tiles, channel tiles, ceil(tiles_m / kTcGroupM)
};

__device__ __forceinline__ uint32_t tc_swizzle(int r) { return (uint32_t)(((r & 1) << 2) ^ ((r >> 1) & 7)); }

// Workgroup id -> tile.  Consecutive workgroup ids go to the eight XCDs in turn, each with its own
// L2: XCD e takes the groups e, e+8, ... of kTcGroupM token tiles and walks a group channel tile
// first, so the workgroups that run on one XCD at a time share a few token tiles and all of W's
// current K-slice.
__device__ __forceinline__ bool tc_tile_of(const TconvArgs &a, int wg, int &tm, int &tn)
{
    const int xcd = wg & 7, seq = wg >> 3;
    const int per_group = kTcGroupM * a.tiles_n;
    const int g = (seq / per_group) * 8 + xcd, in = seq % per_group;
    tm = g * kTcGroupM + in / a.tiles_n;
    tn = in % a.tiles_n;
    return g < a.groups && tm < a.tiles_m;
}

__global__ __launch_bounds__(kThreads) void tconv_mfma(TconvArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    int tm, tn;
    if (!tc_tile_of(a, (int)blockIdx.x, tm, tn)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int M = a.B * a.T * a.HW, D = a.D;
    const int m0 = tm * kTcBM, n0 = tn * kTcBN;
    const int KC = (D + kTcBK - 1) / kTcBK, steps = 3 * KC;

    // ---- loader role: chunk c8 of rows r0 + 32 i ------------------------------------------------
    const int c8 = tid & 7, r0 = tid >> 3;
    int row_t[8], row_c[8];            // frame of the row (or a large value past M), cache row index
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int g = m0 + r0 + 32 * i, gc = g < M ? g : M - 1;
        const int thw = a.T * a.HW, b = gc / thw, rem = gc - b * thw, t = rem / a.HW;
        row_t[i] = g < M ? t : 1 << 20;      // rows past the last token: every tap sees them as past the block
        row_c[i] = b * a.HW + (rem - t * a.HW);
    }
    uint32_t zeroB = 0;                // W rows past the last output channel
#pragma unroll
    for (int i = 0; i < 8; ++i) zeroB |= (n0 + r0 + 32 * i >= D ? 1u : 0u) << i;

    const uint16_t *srcA[8];
    uint32_t zeroA = 0;
    auto set_tap = [&](int tap) {
        zeroA = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ts = row_t[i] + tap - 1;
            const bool front = ts < 0, zero = ts >= a.T || (front && !a.cache);
            const uint16_t *in_x = a.x + ((int64_t)(m0 + r0 + 32 * i) + (int64_t)(tap - 1) * a.HW) * D;
            const uint16_t *in_c = a.cache + (int64_t)row_c[i] * D;
            srcA[i] = zero ? a.x : (front ? in_c : in_x);       // zero rows read some valid row and drop it
            zeroA |= (zero ? 1u : 0u) << i;
        }
    };

    u32x4 stA[8], stB[8];
    bool ktail = false;
    uint32_t zeroA_req = 0;            // zeroA of the step in the staging registers
    // Requests the operand tiles of K-step (tap, kc) into registers.
    auto request = [&](int tap, int kc) {
        int col = kc * kTcBK + c8 * 8;
        ktail = col >= D;
        col = ktail ? 0 : col;
        zeroA_req = zeroA;
        const uint16_t *wrow = a.W + ((int64_t)tap * D + (n0 + r0)) * D + col;
#pragma unroll
        for (int i = 0; i < 8; ++i) stA[i] = *reinterpret_cast<const u32x4 *>(srcA[i] + col);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const bool zr = (zeroB >> i) & 1u;
            stB[i] = *reinterpret_cast<const u32x4 *>(zr ? a.W : wrow + (int64_t)(32 * i) * D);
        }
    };
    const uint32_t wr_off = (uint32_t)r0 * 128u + ((c8 ^ tc_swizzle(r0)) << 4);
    auto deposit = [&](int buf) {
        unsigned char *A = lds + buf * kTcStageBytes, *Bt = A + kTcTileBytes;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const bool zA = ktail || ((zeroA_req >> i) & 1u), zB = ktail || ((zeroB >> i) & 1u);
            *reinterpret_cast<u32x4 *>(A + wr_off + i * 4096) = zA ? zero : stA[i];
            *reinterpret_cast<u32x4 *>(Bt + wr_off + i * 4096) = zB ? zero : stB[i];
        }
    };

    // ---- consumer role ------------------------------------------------------------------------------
    uint32_t ko[4];                    // byte offset of K-chunk pair kk inside the lane's operand row
    {
        const uint32_t g = (uint32_t)(lane >> 5) ^ tc_swizzle(lane & 31);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) ko[kk] = (((uint32_t)kk << 1) ^ g) << 4;
    }
    const uint32_t rdA = (uint32_t)(wm * 128 + (lane & 31)) * 128u, rdB = (uint32_t)(wn * 128 + (lane & 31)) * 128u;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    int tap_n = 0, kc_n = 0;           // the step to request next
    auto advance = [&]() {
        if (++kc_n == KC) {
            kc_n = 0;
            ++tap_n;
            if (tap_n < 3) set_tap(tap_n);
        }
    };
    set_tap(0);
    request(0, 0);
    advance();
    deposit(0);
    __syncthreads();

    auto products = [&](int buf) {
        const unsigned char *A = lds + buf * kTcStageBytes, *Bt = A + kTcTileBytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = *reinterpret_cast<const bf16x8 *>(A + rdA + i * 4096 + ko[kk]);
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = *reinterpret_cast<const bf16x8 *>(Bt + rdB + j * 4096 + ko[kk]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    };
    for (int s = 0; s + 1 < steps; ++s) {
        request(tap_n, kc_n);
        advance();
        products(s & 1);
        deposit((s & 1) ^ 1);
        __syncthreads();
    }
    products((steps - 1) & 1);
    __syncthreads();

    // ---- epilogue: y = bf16(x + acc), 32 token rows of the wave's quadrant at a time through LDS ----
    // (the operand tiles are dead after the loop's last barrier; each wave uses its own region)
    unsigned char *epi = lds + wave * (32 * kTcEpiPitch);
    const int er = lane >> 4, ec = lane & 15;                 // reader: row in a group of four, 8-channel chunk
    const int n = n0 + wn * 128 + ec * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
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
            if (g < M && n < D) {
                const u32x4 xin = *reinterpret_cast<const u32x4 *>(a.x + g * D + n);
                u32x4 out;
                out.x = pack_bf16x2(bf16_lo(xin.x) + lo.x, bf16_hi(xin.x) + lo.y);
                out.y = pack_bf16x2(bf16_lo(xin.y) + lo.z, bf16_hi(xin.y) + lo.w);
                out.z = pack_bf16x2(bf16_lo(xin.z) + hi.x, bf16_hi(xin.z) + hi.y);
                out.w = pack_bf16x2(bf16_lo(xin.w) + hi.z, bf16_hi(xin.w) + hi.w);
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
