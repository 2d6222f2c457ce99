// bf16 MFMA state reduction for d = 64 on gfx950.
//
//   S_c[k][v] = sum_{j in chunk c} phi(K[j][k]) V[j][v],   z_c[k] = sum_{j in chunk c} phi(K[j][k])
//
// (numerator and denominator brackets of the linear-attention equation of
// Sec. 3.2; the per-token state S_j of Sec. 3.3.1 summed over a chunk).
//
// The contraction runs over tokens, but K and V are stored feature-contiguous,
// so both MFMA operands need a transpose.  Each wave works alone on tiles of
// TILE tokens: coalesced 16-byte loads (8 lanes cover one 128-byte token row),
// ReLU on the packed bf16 pairs, a store into the wave's private LDS tile, and
// 32-bit LDS reads down the token axis that are re-packed into operands.  A
// 32-bit word holds features (2r, 2r+1) of one token, so lane r of a 32-row
// MFMA block serves row "feature 2r" in block 0 and "feature 2r+1" in block 1:
// the row/column permutation is undone when the accumulators are written out.
// Because a wave only ever reads LDS it wrote itself, no workgroup barrier is
// needed inside the token loop.
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kRowBytes = 144;   // 128-byte token row + 16 bytes of padding (bank spread, keeps 16-byte alignment)

// Registers of one lane after the loop: the 64x64 fp32 partial state as four
// 32x32 MFMA accumulators, plus 8 key-sum lanes.
struct StateAcc {
    f32x16 s[2][2];   // [row block = key feature parity][col block = value feature parity]
    float z[8];       // features (lane%8)*8 + e of the tokens this lane loaded
};

template <int TILE>
__device__ __forceinline__ void state_tile_load(const uint16_t *Kh, const uint16_t *Vh, int64_t stride_n,
                                                int tok0, int t1, int lane, u32x4 (&kreg)[TILE / 8],
                                                u32x4 (&vreg)[TILE / 8])
{
    const int col = lane & 7;
#pragma unroll
    for (int i = 0; i < TILE / 8; ++i) {
        const int tok = tok0 + (lane >> 3) + 8 * i;
        u32x4 kk = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
        if (tok < t1) {
            kk = *reinterpret_cast<const u32x4 *>(Kh + (int64_t)tok * stride_n + col * 8);
            vv = *reinterpret_cast<const u32x4 *>(Vh + (int64_t)tok * stride_n + col * 8);
        }
        kreg[i] = kk;
        vreg[i] = vv;
    }
}

// Gathers 8 tokens (rows tok_row .. tok_row+7) of 32-bit word `r` from an LDS
// tile and packs the low halves (even feature) and high halves (odd feature)
// into two MFMA operands.
__device__ __forceinline__ void lds_gather_pairs(const unsigned char *tile, int tok_row, int r,
                                                 bf16x8 &even, bf16x8 &odd)
{
    uint32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        w[i] = *reinterpret_cast<const uint32_t *>(tile + (tok_row + i) * kRowBytes + r * 4);
    u32x4 lo, hi;
    lo.x = (w[0] & 0xffffu) | (w[1] << 16);  hi.x = (w[0] >> 16) | (w[1] & 0xffff0000u);
    lo.y = (w[2] & 0xffffu) | (w[3] << 16);  hi.y = (w[2] >> 16) | (w[3] & 0xffff0000u);
    lo.z = (w[4] & 0xffffu) | (w[5] << 16);  hi.z = (w[4] >> 16) | (w[5] & 0xffff0000u);
    lo.w = (w[6] & 0xffffu) | (w[7] << 16);  hi.w = (w[6] >> 16) | (w[7] & 0xffff0000u);
    even = __builtin_bit_cast(bf16x8, lo);
    odd = __builtin_bit_cast(bf16x8, hi);
}

// grid = (C, B*H), block = 256 (4 waves).  Chunk c owns tiles
// [c*T/C, (c+1)*T/C) of the T = ceil((t1-t0)/TILE) tiles; inside the chunk the
// waves take tiles round-robin.  Tokens past t1 are loaded as zeros, which add
// nothing to either sum.  Output: ws[(bh*C + c)][64*64 + 64] fp32, S part in
// [k][v] order.
template <int TILE>
__global__ __launch_bounds__(kThreads, 2) void state_partial_mfma_d64(
    const uint16_t *__restrict__ K, const uint16_t *__restrict__ V, TokStrides st, int H, int t0, int t1,
    int C, float *__restrict__ ws)
{
    static_assert(TILE == 16 || TILE == 32, "tile is one or two MFMA k-steps");
    constexpr int D = 64;
    constexpr int kTileBytes = TILE * kRowBytes;
    constexpr int kSlotFloats = 72 * kWave;                       // 64 S registers + 8 z registers per lane
    constexpr int kStageBytes = kWavesPerWg * 2 * kTileBytes;
    constexpr int kReduceBytes = 2 * kSlotFloats * 4;
    constexpr int kLdsBytes = kStageBytes > kReduceBytes ? kStageBytes : kReduceBytes;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLdsBytes];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const uint16_t *Kh = K + b * st.b + h * st.h;
    const uint16_t *Vh = V + b * st.b + h * st.h;

    const int n_tiles = (t1 - t0 + TILE - 1) / TILE;
    const int tile_lo = chunk_tile_begin(c, C, n_tiles);
    const int tile_hi = chunk_tile_begin(c + 1, C, n_tiles);

    unsigned char *ldsK = lds + wave * 2 * kTileBytes;
    unsigned char *ldsV = ldsK + kTileBytes;

    StateAcc acc;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc.s[rb][cb][i] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc.z[e] = 0.f;

    const int r = lane & 31, g = lane >> 5;
    const int wr_off = (lane >> 3) * kRowBytes + (lane & 7) * 16;

    u32x4 kreg[TILE / 8], vreg[TILE / 8];
    int tile = tile_lo + wave;
    if (tile < tile_hi) state_tile_load<TILE>(Kh, Vh, st.n, t0 + tile * TILE, t1, lane, kreg, vreg);

    for (; tile < tile_hi; tile += kWavesPerWg) {
        // phi(K) on the packed pairs; key sum in fp32 from the same registers
#pragma unroll
        for (int i = 0; i < TILE / 8; ++i) {
            kreg[i] = relu_bf16x8(kreg[i]);
            acc.z[0] += bf16_lo(kreg[i].x);  acc.z[1] += bf16_hi(kreg[i].x);
            acc.z[2] += bf16_lo(kreg[i].y);  acc.z[3] += bf16_hi(kreg[i].y);
            acc.z[4] += bf16_lo(kreg[i].z);  acc.z[5] += bf16_hi(kreg[i].z);
            acc.z[6] += bf16_lo(kreg[i].w);  acc.z[7] += bf16_hi(kreg[i].w);
        }
        wave_lds_fence();   // earlier reads of this tile buffer are done before it is overwritten
#pragma unroll
        for (int i = 0; i < TILE / 8; ++i) {
            *reinterpret_cast<u32x4 *>(ldsK + wr_off + 8 * i * kRowBytes) = kreg[i];
            *reinterpret_cast<u32x4 *>(ldsV + wr_off + 8 * i * kRowBytes) = vreg[i];
        }
        // next tile's loads fly while this one is multiplied
        const int next = tile + kWavesPerWg;
        if (next < tile_hi) state_tile_load<TILE>(Kh, Vh, st.n, t0 + next * TILE, t1, lane, kreg, vreg);
        wave_lds_fence();
#pragma unroll
        for (int s = 0; s < TILE / 16; ++s) {
            bf16x8 a0, a1, b0, b1;
            lds_gather_pairs(ldsK, 16 * s + 8 * g, r, a0, a1);
            lds_gather_pairs(ldsV, 16 * s + 8 * g, r, b0, b1);
            acc.s[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc.s[0][0], 0, 0, 0);
            acc.s[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc.s[0][1], 0, 0, 0);
            acc.s[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc.s[1][0], 0, 0, 0);
            acc.s[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc.s[1][1], 0, 0, 0);
        }
    }

    // ---- combine the four waves in a fixed order: (w0 + w2) + (w1 + w3) --------------------
    float *slot = reinterpret_cast<float *>(lds);
    auto put = [&](float *dst) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int i = 0; i < 16; ++i) dst[((rb * 2 + cb) * 16 + i) * kWave + lane] = acc.s[rb][cb][i];
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[(64 + e) * kWave + lane] = acc.z[e];
    };
    auto add = [&](const float *src) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc.s[rb][cb][i] += src[((rb * 2 + cb) * 16 + i) * kWave + lane];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc.z[e] += src[(64 + e) * kWave + lane];
    };
    __syncthreads();                                   // staging tiles are dead from here on
    if (wave >= 2) put(slot + (wave - 2) * kSlotFloats);
    __syncthreads();
    if (wave < 2) add(slot + wave * kSlotFloats);
    __syncthreads();
    if (wave == 1) put(slot);
    __syncthreads();
    if (wave != 0) return;
    add(slot);

    // ---- wave 0 writes the chunk's partial state in [k][v] order ----------------------------
    // 32x32 accumulator layout: register i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32.
    float *out = ws + ((int64_t)bh * C + c) * (D * D + D);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = 8 * (i >> 2) + 4 * g + (i & 3);
            const int k = 2 * m + rb;
            f32x2 pair = {acc.s[rb][0][i], acc.s[rb][1][i]};       // value features 2r, 2r+1
            *reinterpret_cast<f32x2 *>(out + k * D + 2 * r) = pair;
        }
    // key sum: lanes with equal lane%8 hold the same 8 features
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float x = acc.z[e];
        x += __shfl_xor(x, 8);
        x += __shfl_xor(x, 16);
        x += __shfl_xor(x, 32);
        acc.z[e] = x;
    }
    if (lane < 8) {
        f32x4 lo = {acc.z[0], acc.z[1], acc.z[2], acc.z[3]};
        f32x4 hi = {acc.z[4], acc.z[5], acc.z[6], acc.z[7]};
        *reinterpret_cast<f32x4 *>(out + D * D + lane * 8) = lo;
        *reinterpret_cast<f32x4 *>(out + D * D + lane * 8 + 4) = hi;
    }
}

}  // namespace sv
