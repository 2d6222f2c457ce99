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
// operand; every wave loads it once, straight from global memory, splits each
// fp32 value into a bf16 hi + lo pair (S = hi + lo to ~2^-17) and keeps it in
// registers for its whole token range.  The key sum z rides along as two extra
// operand rows (hi and lo), so the denominator comes out of the same MFMA pass
// in fp32 and only has to be handed to the lane that holds the token's other
// 32 features (one cross-lane exchange).  phi(Q)^T is the B operand: a lane
// needs 8 consecutive features of one token, i.e. 16 contiguous bytes of the
// token row.  Q tiles come in with coalesced non-temporal 16-byte loads and
// pass through a wave-private LDS tile to reach that layout; O tiles go back
// through the same tile so that stores are coalesced too.  No workgroup
// barrier is needed anywhere.
#pragma once

#include "common.hpp"
#include "state_mfma.hpp"   // kRowBytes
#include "sync.hpp"

namespace sv {

constexpr int kApplyTile = 32;   // tokens per wave tile (the N dimension of the 32x32x16 MFMA)

__device__ __forceinline__ void apply_tile_load(const uint16_t *Qh, int64_t stride_n, int tok0, int t1, int lane,
                                                u32x4 (&qreg)[kApplyTile / 8])
{
    const int col = lane & 7;
#pragma unroll
    for (int i = 0; i < kApplyTile / 8; ++i) {
        const int tok = tok0 + (lane >> 3) + 8 * i;
        u32x4 q = {0u, 0u, 0u, 0u};
        if (tok < t1) q = load_stream16(Qh + (int64_t)tok * stride_n + col * 8);
        qreg[i] = q;
    }
}

// The state of one head as MFMA A operands, per lane (m = lane%32, g = lane/32).
//   S rows: MFMA row m of row block rb stands for output feature
//     F(rb, m) = 32*((m/4)%2) + 16*rb + 4*(m/8) + m%4,
//   chosen so that accumulator register i of a lane in half g' = lane/32 is
//   output feature 32*g' + 16*rb + i of the lane's token.
//   z rows: row 0 = hi(z), row 1 = lo(z), rows 2..31 = 0.
template <bool HILO>
struct ApplyOperands {
    static constexpr int NS = HILO ? 2 : 1;
    bf16x8 s[NS][2][4];    // [hi/lo][row block][k-step]
    bf16x8 zrow[4];        // [k-step]

    // COHERENT: the state was written by another workgroup of this same kernel.
    template <bool COHERENT>
    __device__ __forceinline__ void load(const float *__restrict__ Sh, const float *__restrict__ zh, int lane)
    {
        const int m = lane & 31, g = lane >> 5;
        float sv_[2][4][8];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int F = 32 * ((m >> 2) & 1) + 16 * rb + 4 * (m >> 3) + (m & 3);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float *p = Sh + (16 * ks + 8 * g + i) * 64 + F;
                    sv_[rb][ks][i] = COHERENT ? load_coherent1(p) : *p;
                }
        }
        float zv[4][8];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float *p = zh + 16 * ks + 8 * g + i;
                zv[ks][i] = COHERENT ? load_coherent1(p) : *p;
            }
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const float a = sv_[rb][ks][2 * p], b = sv_[rb][ks][2 * p + 1];
                    hi[p] = pack_bf16x2(a, b);
                    lo[p] = pack_bf16x2(a - bf16_lo(hi[p]), b - bf16_hi(hi[p]));
                }
                const u32x4 h4 = {hi[0], hi[1], hi[2], hi[3]}, l4 = {lo[0], lo[1], lo[2], lo[3]};
                s[0][rb][ks] = __builtin_bit_cast(bf16x8, h4);
                if (HILO) s[NS - 1][rb][ks] = __builtin_bit_cast(bf16x8, l4);
            }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint32_t w[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float a = zv[ks][2 * p], b = zv[ks][2 * p + 1];
                const uint32_t hi = pack_bf16x2(a, b);
                const uint32_t lo = pack_bf16x2(a - bf16_lo(hi), b - bf16_hi(hi));
                w[p] = m == 0 ? hi : (m == 1 ? lo : 0u);
            }
            const u32x4 w4 = {w[0], w[1], w[2], w[3]};
            zrow[ks] = __builtin_bit_cast(bf16x8, w4);
        }
    }
};

// One wave's share of the token range [t0, t1): tiles first_tile, first_tile +
// tile_step, ... below n_tiles (32 tokens each).  `tileQ` is this wave's private
// LDS tile (kApplyTile * kRowBytes bytes).  `qreg` holds the first DEPTH tiles,
// already requested by the caller with apply_prefetch (stages FROM..TO-1 per call).
template <int DEPTH, int FROM = 0, int TO = DEPTH>
__device__ __forceinline__ void apply_prefetch(const uint16_t *Qh, int64_t stride_n, int t0, int t1, int first_tile,
                                               int tile_step, int n_tiles, int lane,
                                               u32x4 (&qreg)[DEPTH][kApplyTile / 8])
{
#pragma unroll
    for (int s = FROM; s < TO; ++s) {
        const int t = first_tile + s * tile_step;
        if (t < n_tiles) apply_tile_load(Qh, stride_n, t0 + t * kApplyTile, t1, lane, qreg[s]);
    }
}

// ROPE: the numerator uses queries rotated after the ReLU (table row = token index); the
// denominator keeps the plain ones.  The wave's LDS region then holds a second,
// rotated copy of each tile after the NB plain ones, and `rope` is the table.
template <bool HILO, int DEPTH, int NB, bool ROPE>
__device__ __forceinline__ void apply_tiles(const uint16_t *Qh, uint16_t *Oh, const float *rope, int64_t stride_n,
                                            int t0, int t1, int first_tile, int tile_step, int n_tiles,
                                            unsigned char *tileQ, int lane, const ApplyOperands<HILO> &A, float eps,
                                            u32x4 (&qreg)[DEPTH][kApplyTile / 8])
{
    static_assert(DEPTH % NB == 0, "stages are consumed NB at a time");
    static_assert(!ROPE || (NB == 1 && DEPTH % 2 == 0), "the table ring below alternates between two slots");
    constexpr int NS = HILO ? 2 : 1;
    constexpr int kTileBytes = kApplyTile * kRowBytes;
    const int n = lane & 31, g = lane >> 5;
    const int wr_off = (lane >> 3) * kRowBytes + (lane & 7) * 16;

    // rotation-table entries of the tile in work and of the next one (slot = stage parity)
    f32x4 cs[ROPE ? 2 : 1][kApplyTile / 8][2];
    if (ROPE && first_tile < n_tiles) rope_tile_load<kApplyTile>(rope, t0 + first_tile * kApplyTile, t1, lane, cs[0]);

    // NB tiles go through each phase together, so that one tile's LDS and
    // conversion latencies hide behind the other's MFMA chain.
    int tile = first_tile;
    while (tile < n_tiles) {
#pragma unroll
        for (int s0 = 0; s0 < DEPTH; s0 += NB) {
            if (tile < n_tiles) {
                bool valid[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) valid[j] = tile + j * tile_step < n_tiles;

                wave_lds_fence();
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (valid[j]) {
#pragma unroll
                        for (int i = 0; i < kApplyTile / 8; ++i) {
                            const u32x4 pq = relu_bf16x8(qreg[s0 + j][i]);                          // phi(Q)
                            *reinterpret_cast<u32x4 *>(tileQ + j * kTileBytes + wr_off + 8 * i * kRowBytes) = pq;
                            if (ROPE)
                                *reinterpret_cast<u32x4 *>(tileQ + (NB + j) * kTileBytes + wr_off + 8 * i * kRowBytes) =
                                    rope_rotate_bf16x8(pq, cs[ROPE ? s0 & 1 : 0][i][0], cs[ROPE ? s0 & 1 : 0][i][1]);
                        }
                        const int nxt = tile + (j + DEPTH) * tile_step;
                        if (nxt < n_tiles)
                            apply_tile_load(Qh, stride_n, t0 + nxt * kApplyTile, t1, lane, qreg[s0 + j]);
                        if (ROPE && tile + tile_step < n_tiles)
                            rope_tile_load<kApplyTile>(rope, t0 + (tile + tile_step) * kApplyTile, t1, lane,
                                                       cs[ROPE ? (s0 & 1) ^ 1 : 0]);
                    }
                wave_lds_fence();

                // B operands: features 16*ks + 8g .. +8 of token n (Br: the rotated copy for the numerator)
                bf16x8 Bq[NB][4], Br[ROPE ? NB : 1][4];
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (valid[j]) {
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) {
                            Bq[j][ks] = *reinterpret_cast<const bf16x8 *>(tileQ + j * kTileBytes + n * kRowBytes +
                                                                          (16 * ks + 8 * g) * 2);
                            if (ROPE)
                                Br[j][ks] = *reinterpret_cast<const bf16x8 *>(tileQ + (NB + j) * kTileBytes +
                                                                              n * kRowBytes + (16 * ks + 8 * g) * 2);
                        }
                    }

                f32x16 acc[NB][2], accz[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int i = 0; i < 16; ++i) { acc[j][0][i] = 0.f; acc[j][1][i] = 0.f; accz[j][i] = 0.f; }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        if (valid[j])
                            accz[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.zrow[ks], Bq[j][ks], accz[j], 0, 0, 0);
#pragma unroll
                for (int p = NS - 1; p >= 0; --p)      // small (lo) terms first
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                        for (int j = 0; j < NB; ++j)
                            if (valid[j]) {
                                const bf16x8 bq = ROPE ? Br[ROPE ? j : 0][ks] : Bq[j][ks];
                                acc[j][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.s[p][0][ks], bq, acc[j][0], 0, 0, 0);
                                acc[j][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.s[p][1][ks], bq, acc[j][1], 0, 0, 0);
                            }

                wave_lds_fence();
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (valid[j]) {
                        // denominator: rows 0 (hi) and 1 (lo) of the z block sit in registers 0 and 1 of
                        // the lanes of the lower half; the upper half fetches them across the wave
                        float den = accz[j][1] + accz[j][0];
                        den = __shfl(den, n);
                        const float inv = 1.0f / (den + eps);
#pragma unroll
                        for (int rb = 0; rb < 2; ++rb) {
                            const f32x16 &a = acc[j][rb];
                            u32x4 lo4, hi4;
                            lo4.x = pack_bf16x2(a[0] * inv, a[1] * inv);
                            lo4.y = pack_bf16x2(a[2] * inv, a[3] * inv);
                            lo4.z = pack_bf16x2(a[4] * inv, a[5] * inv);
                            lo4.w = pack_bf16x2(a[6] * inv, a[7] * inv);
                            hi4.x = pack_bf16x2(a[8] * inv, a[9] * inv);
                            hi4.y = pack_bf16x2(a[10] * inv, a[11] * inv);
                            hi4.z = pack_bf16x2(a[12] * inv, a[13] * inv);
                            hi4.w = pack_bf16x2(a[14] * inv, a[15] * inv);
                            unsigned char *row = tileQ + j * kTileBytes + n * kRowBytes + (32 * g + 16 * rb) * 2;
                            *reinterpret_cast<u32x4 *>(row) = lo4;
                            *reinterpret_cast<u32x4 *>(row + 16) = hi4;
                        }
                    }
                wave_lds_fence();
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    if (valid[j]) {
                        const int tok0 = t0 + (tile + j * tile_step) * kApplyTile;
#pragma unroll
                        for (int i = 0; i < kApplyTile / 8; ++i) {
                            const int tok = tok0 + (lane >> 3) + 8 * i;
                            const u32x4 o = *reinterpret_cast<const u32x4 *>(tileQ + j * kTileBytes + wr_off +
                                                                             8 * i * kRowBytes);
                            if (tok < t1) store_stream16(Oh + (int64_t)tok * stride_n + (lane & 7) * 8, o);
                        }
                    }
            }
            tile += NB * tile_step;
        }
    }
}

// LDS bytes per wave and in total: NB tiles, twice that with ROPE (plain + rotated copies).
template <int NB, bool ROPE>
__host__ __device__ constexpr int apply_wave_lds_bytes() { return (ROPE ? 2 : 1) * NB * kApplyTile * kRowBytes; }
template <int WAVES, int NB, bool ROPE>
__host__ __device__ constexpr int apply_lds_bytes() { return WAVES * apply_wave_lds_bytes<NB, ROPE>(); }

// grid = (C, B*H), block = 64*WAVES.  Wave w of workgroup c owns tiles
// WAVES*c + w + WAVES*C*i (i = 0, 1, ...) of the T = ceil((t1-t0)/32) tiles,
// the same round-robin deal as the state kernel.
// HILO = false drops the low half of S (one MFMA pass instead of two).
// NB tiles of a wave are in the arithmetic phase together.
template <bool HILO, int WAVES, int DEPTH, int NB, bool ROPE>
__global__ __launch_bounds__(64 * WAVES, 1) void apply_mfma_d64(
    const uint16_t *__restrict__ Q, uint16_t *__restrict__ O, const float *__restrict__ rope, TokStrides st, int H,
    int t0, int t1, int C, const float *__restrict__ S, const float *__restrict__ z, float eps)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const uint16_t *Qh = Q + b * st.b + h * st.h;
    uint16_t *Oh = O + b * st.b + h * st.h;
    const int n_tiles = (t1 - t0 + kApplyTile - 1) / kApplyTile;
    const int first = WAVES * c + wave, step = WAVES * C;

    u32x4 qreg[DEPTH][kApplyTile / 8];
    apply_prefetch<DEPTH>(Qh, st.n, t0, t1, first, step, n_tiles, lane, qreg);   // in flight while S is fetched
    ApplyOperands<HILO> A;
    A.template load<false>(S + (size_t)bh * 64 * 64, z + (size_t)bh * 64, lane);
    apply_tiles<HILO, DEPTH, NB, ROPE>(Qh, Oh, rope, st.n, t0, t1, first, step, n_tiles,
                                       lds + wave * apply_wave_lds_bytes<NB, ROPE>(), lane, A, eps, qreg);
}

}  // namespace sv
