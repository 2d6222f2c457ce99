// bf16 MFMA apply for d = 64 on gfx950.
//
//   O[i][v] = (sum_k phi(Q[i][k]) S[k][v]) / (sum_k phi(Q[i][k]) z[k] + eps)
//
// (right-hand form of the linear-attention equation of Sec. 3.2; first equality
// of the causal re-formulation in Sec. 3.3.1).
//
// The product is computed transposed, O^T = S^T phi(Q)^T, so that the token
// axis lands on the lanes of the accumulator: each lane ends up with 32
// consecutive output features of ONE token and can normalise them with that
// token's denominator and pack them into 64 contiguous bytes.  S^T is the A
// operand; it is converted once per workgroup from fp32 into a bf16 hi + lo
// pair (S = hi + lo to ~2^-17), staged through LDS, and then lives in registers
// for the workgroup's whole token range.  phi(Q)^T is the B operand: a lane
// needs 8 consecutive features of one token, i.e. 16 contiguous bytes of the
// token row.  Q tiles come in with coalesced 16-byte loads and pass through a
// wave-private LDS tile to reach that layout; O tiles go back through the same
// tile so that stores are coalesced too.  The denominator is a per-lane fp32
// dot product over the lane's 32 features, completed by one cross-lane exchange
// with the lane that holds the token's other 32 features.
#pragma once

#include "common.hpp"
#include "state_mfma.hpp"   // kRowBytes

namespace sv {

template <int TILE>
__device__ __forceinline__ void apply_tile_load(const uint16_t *Qh, int64_t stride_n, int tok0, int t1, int lane,
                                                u32x4 (&qreg)[TILE / 8])
{
    const int col = lane & 7;
#pragma unroll
    for (int i = 0; i < TILE / 8; ++i) {
        const int tok = tok0 + (lane >> 3) + 8 * i;
        u32x4 q = {0u, 0u, 0u, 0u};
        if (tok < t1) q = *reinterpret_cast<const u32x4 *>(Qh + (int64_t)tok * stride_n + col * 8);
        qreg[i] = q;
    }
}

// grid = (C, B*H), block = 256 (4 waves).  Chunk c owns tiles [c*T/C, (c+1)*T/C)
// of the T = ceil((t1-t0)/32) tiles of 32 tokens; waves take tiles round-robin.
// HILO = false drops the low half of S (one MFMA pass instead of two).
template <bool HILO>
__global__ __launch_bounds__(kThreads, 2) void apply_mfma_d64(
    const uint16_t *__restrict__ Q, uint16_t *__restrict__ O, TokStrides st, int H, int t0, int t1, int C,
    const float *__restrict__ S, const float *__restrict__ z, float eps)
{
    constexpr int D = 64;
    constexpr int TILE = 32;
    constexpr int NS = HILO ? 2 : 1;
    constexpr int kTileBytes = TILE * kRowBytes;
    constexpr int kStBytes = D * kRowBytes;                       // one transposed bf16 copy of S
    constexpr int kPrologueBytes = NS * kStBytes;
    constexpr int kStageBytes = kWavesPerWg * kTileBytes;
    constexpr int kLdsBytes = kPrologueBytes > kStageBytes ? kPrologueBytes : kStageBytes;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLdsBytes];
    __shared__ __attribute__((aligned(16))) float sz[D];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const uint16_t *Qh = Q + b * st.b + h * st.h;
    uint16_t *Oh = O + b * st.b + h * st.h;

    const int n_tiles = (t1 - t0 + TILE - 1) / TILE;
    const int tile_lo = chunk_tile_begin(c, C, n_tiles);
    const int tile_hi = chunk_tile_begin(c + 1, C, n_tiles);

    // first Q tile is requested before the state is staged
    u32x4 qreg[TILE / 8];
    int tile = tile_lo + wave;
    if (tile < tile_hi) apply_tile_load<TILE>(Qh, st.n, t0 + tile * TILE, t1, lane, qreg);

    // ---- stage S^T as bf16 hi (+ lo): st[v][k], rows padded to kRowBytes --------------------
    {
        const float *Sh = S + (int64_t)bh * D * D;
        for (int idx = tid; idx < D * D; idx += kThreads) {
            const int k = idx >> 6, v = idx & 63;
            const float s = Sh[idx];
            const uint16_t hi = f32_to_bf16_bits(s);
            *reinterpret_cast<uint16_t *>(lds + v * kRowBytes + k * 2) = hi;
            if (HILO) {
                const uint16_t lo = f32_to_bf16_bits(s - bf16_bits_to_f32(hi));
                *reinterpret_cast<uint16_t *>(lds + kStBytes + v * kRowBytes + k * 2) = lo;
            }
        }
        if (tid < D) sz[tid] = z[(int64_t)bh * D + tid];
    }
    __syncthreads();

    // A operands: MFMA row m of row block rb stands for output feature
    //   F(rb, m) = 32*((m/4)%2) + 16*rb + 4*(m/8) + m%4,
    // chosen so that accumulator register i of a lane in half g' = lane/32 is
    // output feature 32*g' + 16*rb + i of the lane's token.
    const int n = lane & 31, g = lane >> 5;
    bf16x8 A[NS][2][4];
    {
        const int m = n;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int F = 32 * ((m >> 2) & 1) + 16 * rb + 4 * (m >> 3) + (m & 3);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int p = 0; p < NS; ++p)
                    A[p][rb][s] = *reinterpret_cast<const bf16x8 *>(lds + p * kStBytes + F * kRowBytes +
                                                                    (16 * s + 8 * g) * 2);
        }
    }
    __syncthreads();   // the prologue region is reused as Q/O staging below

    unsigned char *ldsQ = lds + wave * kTileBytes;
    const int wr_off = (lane >> 3) * kRowBytes + (lane & 7) * 16;

    for (; tile < tile_hi; tile += kWavesPerWg) {
        const int tok0 = t0 + tile * TILE;
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < TILE / 8; ++i)
            *reinterpret_cast<u32x4 *>(ldsQ + wr_off + 8 * i * kRowBytes) = relu_bf16x8(qreg[i]);   // phi(Q)
        const int next = tile + kWavesPerWg;
        if (next < tile_hi) apply_tile_load<TILE>(Qh, st.n, t0 + next * TILE, t1, lane, qreg);
        wave_lds_fence();

        // B operands: features 16s + 8g .. +8 of token n
        u32x4 Bq[4];
#pragma unroll
        for (int s = 0; s < 4; ++s)
            Bq[s] = *reinterpret_cast<const u32x4 *>(ldsQ + n * kRowBytes + (16 * s + 8 * g) * 2);

        // denominator: this lane's 32 features, then the other half of the token
        float den = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const f32x4 z0 = *reinterpret_cast<const f32x4 *>(sz + 16 * s + 8 * g);
            const f32x4 z1 = *reinterpret_cast<const f32x4 *>(sz + 16 * s + 8 * g + 4);
            den = fmaf(bf16_lo(Bq[s].x), z0.x, den);  den = fmaf(bf16_hi(Bq[s].x), z0.y, den);
            den = fmaf(bf16_lo(Bq[s].y), z0.z, den);  den = fmaf(bf16_hi(Bq[s].y), z0.w, den);
            den = fmaf(bf16_lo(Bq[s].z), z1.x, den);  den = fmaf(bf16_hi(Bq[s].z), z1.y, den);
            den = fmaf(bf16_lo(Bq[s].w), z1.z, den);  den = fmaf(bf16_hi(Bq[s].w), z1.w, den);
        }
        den += __shfl_xor(den, 32);

        f32x16 acc[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;
#pragma unroll
            for (int p = NS - 1; p >= 0; --p)      // small (lo) terms first
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        A[p][rb][s], __builtin_bit_cast(bf16x8, Bq[s]), acc[rb], 0, 0, 0);
        }

        // normalise, round to bf16, and send the tile back through LDS
        const float inv = 1.0f / (den + eps);
        wave_lds_fence();
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            u32x4 lo4, hi4;
            lo4.x = pack_bf16x2(acc[rb][0] * inv, acc[rb][1] * inv);
            lo4.y = pack_bf16x2(acc[rb][2] * inv, acc[rb][3] * inv);
            lo4.z = pack_bf16x2(acc[rb][4] * inv, acc[rb][5] * inv);
            lo4.w = pack_bf16x2(acc[rb][6] * inv, acc[rb][7] * inv);
            hi4.x = pack_bf16x2(acc[rb][8] * inv, acc[rb][9] * inv);
            hi4.y = pack_bf16x2(acc[rb][10] * inv, acc[rb][11] * inv);
            hi4.z = pack_bf16x2(acc[rb][12] * inv, acc[rb][13] * inv);
            hi4.w = pack_bf16x2(acc[rb][14] * inv, acc[rb][15] * inv);
            unsigned char *row = ldsQ + n * kRowBytes + (32 * g + 16 * rb) * 2;
            *reinterpret_cast<u32x4 *>(row) = lo4;
            *reinterpret_cast<u32x4 *>(row + 16) = hi4;
        }
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < TILE / 8; ++i) {
            const int tok = tok0 + (lane >> 3) + 8 * i;
            const u32x4 o = *reinterpret_cast<const u32x4 *>(ldsQ + wr_off + 8 * i * kRowBytes);
            if (tok < t1) *reinterpret_cast<u32x4 *>(Oh + (int64_t)tok * st.n + (lane & 7) * 8) = o;
        }
    }
}

}  // namespace sv
