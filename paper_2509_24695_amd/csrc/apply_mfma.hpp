// bf16 MFMA apply for d = 64, 112 and 128 on gfx950.
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
// 32 features (one cross-lane exchange); DEN_VALU takes it on the vector ALU
// instead (a wavefront-level reduction), which measures level.  phi(Q)^T is the B operand: a lane
// needs 8 consecutive features of one token, i.e. 16 contiguous bytes of the
// token row.  Q tiles come in with coalesced non-temporal 16-byte loads and
// pass through a wave-private LDS tile to reach that layout; O tiles go back
// through the same tile so that stores are coalesced too.  No workgroup
// barrier is needed anywhere.  On this hardware loads and stores share one
// in-order completion counter, and every stage issues a fixed number of both, so
// a tile waits only for its own loads: the stores of earlier tiles and the loads
// of later ones stay in flight.
//
// d = 112 and 128: a wave produces 64 of a token's output features (value
// block vb), so it keeps a 128 x 64 panel of S in registers (ApplyOperands<128>)
// and runs twice as many k-steps; the token streaming for that case is in
// coop128.hpp.
#pragma once

#include "common.hpp"
#include "state_mfma.hpp"   // TileWalk, kOutOfRange handling
#include "sync.hpp"

namespace sv {

constexpr int kApplyTile = 32;   // tokens per wave tile (the N dimension of the 32x32x16 MFMA)

// The state of one head as MFMA A operands for the 32*NB output features of value
// block vb, per lane (m = lane%32, g = lane/32).
//   S rows: MFMA row m of row block rb stands for output feature
//     32*NB*vb + F(rb, m),  F(rb, m) = 16*NB*((m/4)%2) + 16*rb + 4*(m/8) + m%4,
//   chosen so that accumulator register i of a lane in half g' = lane/32 is
//   output feature 32*NB*vb + 16*NB*g' + 16*rb + i of the lane's token (NB = 2: 32
//   consecutive features per lane, NB = 1: 16).
//   z rows: row 0 = hi(z), row 1 = lo(z), rows 2..31 = 0.
// The contraction runs over DP key features in DP/16 k-steps; S is d x d (row
// length d) and z has d entries, anything past d counts as zero.
// ZROWS = false leaves the z rows out (the caller takes the denominators another way).
template <int DP, bool HILO, int NB = 2, bool ZROWS = true>
struct ApplyOperands {
    static constexpr int NS = HILO ? 2 : 1;
    static constexpr int KS = DP / 16;
    bf16x8 s[NS][NB][KS];          // [hi/lo][row block][k-step]
    bf16x8 zrow[ZROWS ? KS : 1];   // [k-step]

    // LDS that load_shared stages through: the operand words of S, then the hi and lo words of the z rows.
    static constexpr int kSharedStateBytes = 2 * NB * KS * 64 * 16, kSharedBytes = kSharedStateBytes + KS * 2 * 2 * 16;

    // The same operands (DP = 64, value block 0), fetched once per workgroup instead of once per wave:
    // wave w converts k-step w of S and of the two z rows and hands them round through `stage`
    // (kSharedBytes of LDS, free again when this returns).  Must be called by all four waves.  COHERENT: the state was written by another workgroup of this same kernel.
    template <bool COHERENT>
    __device__ __forceinline__ void load_shared(const float *__restrict__ Sh, const float *__restrict__ zh, int wave,
                                                int lane, unsigned char *stage)
    {
        static_assert(DP == 64 && ZROWS, "the d = 64 apply kernel");
        bf16x8 *st = reinterpret_cast<bf16x8 *>(stage);       // [hi/lo][row block][k-step][lane]
        const int m = lane & 31, g = lane >> 5;
        // every load of the function goes out before the first value is looked at: one memory round trip, not one
        // per row block and one for the key sums (the compiler keeps coherent loads in program order)
        float sa[NB][8];
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            const int F = 16 * NB * ((m >> 2) & 1) + 16 * rb + 4 * (m >> 3) + (m & 3);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = 16 * wave + 8 * g + i;
                sa[rb][i] = COHERENT ? load_coherent1(Sh + k * 64 + F) : Sh[k * 64 + F];
            }
        }
        float zv[8];                                          // the key sums of k-step `wave`
#pragma unroll
        for (int i = 0; i < 8; ++i) zv[i] = COHERENT ? load_coherent1(zh + 16 * wave + 8 * g + i) : zh[16 * wave + 8 * g + i];
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float a = sa[rb][2 * p], b = sa[rb][2 * p + 1];
                hi[p] = pack_bf16x2(a, b);
                lo[p] = pack_bf16x2(a - bf16_lo(hi[p]), b - bf16_hi(hi[p]));
            }
            const u32x4 h4 = {hi[0], hi[1], hi[2], hi[3]}, l4 = {lo[0], lo[1], lo[2], lo[3]};
            st[((0 * NB + rb) * KS + wave) * 64 + lane] = __builtin_bit_cast(bf16x8, h4);
            st[((1 * NB + rb) * KS + wave) * 64 + lane] = __builtin_bit_cast(bf16x8, l4);
        }
        // z rows: the hi and lo words of k-step `wave`, once per half wave: [k-step][g][hi/lo] behind the S words
        u32x4 *zst = reinterpret_cast<u32x4 *>(stage + kSharedStateBytes);
        {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float a = zv[2 * p], b = zv[2 * p + 1];
                hi[p] = pack_bf16x2(a, b);
                lo[p] = pack_bf16x2(a - bf16_lo(hi[p]), b - bf16_hi(hi[p]));
            }
            if (m == 0) {
                zst[(wave * 2 + g) * 2 + 0] = u32x4{hi[0], hi[1], hi[2], hi[3]};
                zst[(wave * 2 + g) * 2 + 1] = u32x4{lo[0], lo[1], lo[2], lo[3]};
            }
        }
        wg_barrier();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) {
                s[0][rb][ks] = st[((0 * NB + rb) * KS + ks) * 64 + lane];
                if (HILO) s[NS - 1][rb][ks] = st[((1 * NB + rb) * KS + ks) * 64 + lane];
            }
            const u32x4 w4 = zst[(ks * 2 + g) * 2 + (m & 1)];            // row 0 = hi(z), row 1 = lo(z), the rest 0
            zrow[ks] = __builtin_bit_cast(bf16x8, m < 2 ? w4 : u32x4{0u, 0u, 0u, 0u});
        }
        wg_barrier();                        // `stage` may be written again
    }

    // COHERENT: the state was written by another workgroup of this same kernel.
    template <bool COHERENT>
    __device__ __forceinline__ void load(const float *__restrict__ Sh, const float *__restrict__ zh, int d, int vb,
                                         int lane)
    {
        const int m = lane & 31, g = lane >> 5;
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            const int F = 32 * NB * vb + 16 * NB * ((m >> 2) & 1) + 16 * rb + 4 * (m >> 3) + (m & 3);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                // every lane loads (a valid address where its element does not exist) and the value is dropped
                // afterwards: a load under a condition becomes a branch, and the compiler then waits for each
                // load before the next branch - eight dependent round trips instead of one
                float sv_[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int k = 16 * ks + 8 * g + i;
                    const bool exists = DP == 64 || (k < d && F < d);
                    const float *p = Sh + (exists ? k * d + F : 0);
                    const float x = COHERENT ? load_coherent1(p) : *p;
                    sv_[i] = exists ? x : 0.f;
                }
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const float a = sv_[2 * p], b = sv_[2 * p + 1];
                    hi[p] = pack_bf16x2(a, b);
                    lo[p] = pack_bf16x2(a - bf16_lo(hi[p]), b - bf16_hi(hi[p]));
                }
                const u32x4 h4 = {hi[0], hi[1], hi[2], hi[3]}, l4 = {lo[0], lo[1], lo[2], lo[3]};
                s[0][rb][ks] = __builtin_bit_cast(bf16x8, h4);
                if (HILO) s[NS - 1][rb][ks] = __builtin_bit_cast(bf16x8, l4);
            }
        }
#pragma unroll
        for (int ks = 0; ks < (ZROWS ? KS : 0); ++ks) {
            uint32_t w[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int k = 16 * ks + 8 * g + 2 * p;
                const bool exists = DP == 64 || k < d;       // d is even: k and k + 1 exist together
                const float *pz = zh + (exists ? k : 0);
                float a = COHERENT ? load_coherent1(pz) : pz[0];
                float b = COHERENT ? load_coherent1(pz + 1) : pz[1];
                a = exists ? a : 0.f;
                b = exists ? b : 0.f;
                const uint32_t hi = pack_bf16x2(a, b);
                const uint32_t lo = pack_bf16x2(a - bf16_lo(hi), b - bf16_hi(hi));
                w[p] = m == 0 ? hi : (m == 1 ? lo : 0u);
            }
            const u32x4 w4 = {w[0], w[1], w[2], w[3]};
            zrow[ks] = __builtin_bit_cast(bf16x8, w4);
        }
    }
};

// The key sums a lane needs when the denominators are taken on the vector ALU (DEN_VALU): those of the 32
// features of a token that pass through the lane as B operands, zf[ks][e] = z[16 ks + 8 (lane / 32) + e].
template <bool COHERENT>
__device__ __forceinline__ void load_key_sums(const float *__restrict__ zh, int lane, float (&zf)[4][8])
{
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float *p = zh + 16 * ks + 8 * (lane >> 5) + e;
            zf[ks][e] = COHERENT ? load_coherent1(p) : *p;
        }
}

// One wave's token stream (d = 64): buffer resources over the head's Q and O
// rows below the end of the token range, the wave's tile walk (32 tokens per
// tile), the register staging of DEPTH tiles in flight, and the rotation source.
template <int DEPTH, int ROPE>
struct ApplyStream {
    rsrc_t rQ, rO;
    uint32_t row_bytes, lane_off;
    TileWalk walk;
    u32x4 q[DEPTH][kApplyTile / 8];
    Rotator<ROPE, kApplyTile / 8, DEPTH> rot;

    __device__ __forceinline__ ApplyStream(const uint16_t *Qh, uint16_t *Oh, const RopeArg &rope,
                                           const unsigned char *lds_tab, int64_t stride_n, int t1, int lane,
                                           const TileWalk &w)
        : rQ(make_rsrc(Qh, (uint32_t)t1 * (uint32_t)stride_n * 2u)),
          rO(make_rsrc(Oh, (uint32_t)t1 * (uint32_t)stride_n * 2u)), row_bytes((uint32_t)stride_n * 2u),
          lane_off((uint32_t)(lane >> 3) * (uint32_t)stride_n * 2u + (uint32_t)(lane & 7) * 16u), walk(w),
          rot(rope, t1, 64, lane >> 3, 8, 4 * (lane & 7), 1, lds_tab) {}

    // Requests the wave's i-th tile into stage s; past the share nothing is read.
    __device__ __forceinline__ void request(int s, int i)
    {
        const uint32_t base = walk.offset<kApplyTile>(i, row_bytes);
#pragma unroll
        for (int j = 0; j < kApplyTile / 8; ++j)
            q[s][j] = load_stream16(rQ, base + lane_off + (uint32_t)j * 8u * row_bytes);
        rot.request(s, i < walk.count, walk.token<kApplyTile>(i));
    }
};

// Requests tiles FROM .. TO-1 of the wave's share into the stages of the same numbers.
template <int FROM, int TO, int DEPTH, int ROPE>
__device__ __forceinline__ void apply_prefetch(ApplyStream<DEPTH, ROPE> &st)
{
#pragma unroll
    for (int s = FROM; s < TO; ++s) {
        st.request(s, s);
        __builtin_amdgcn_sched_barrier(0);   // requests go out in stage order, as they do in the loop
    }
}

// Applies the state in `A` to the wave's share, whose first DEPTH tiles
// apply_prefetch has requested.  `tileQ` is this wave's private LDS region: one
// tile of kApplyTile rows of kRowBytes bytes, two with ROPE (the
// numerator then uses queries rotated after the ReLU, the denominator the plain
// ones).  Tiles are taken DEPTH at a time; every stage issues its loads and
// stores whether or not it still has a tile (out of range they do nothing), only
// the arithmetic is skipped.
//
// Two measurement variants (sv_measure_apply_variant; the library's own calls use neither):
//   S_LDS     the operands of S stay in LDS (`s_lds`: the layout load_shared stages them in, shared by the
//             workgroup's waves) and are read again for every tile, instead of living in each wave's registers;
//   DEN_VALU  the denominators are taken on the vector ALU - every lane multiplies the 32 features of its token
//             that pass through it as B operands with their key sums (`zf`, [k-step][feature]) and the two
//             half-waves exchange their halves - instead of riding through the matrix core as two operand rows.
template <bool HILO, int DEPTH, int ROPE, bool S_LDS = false, bool DEN_VALU = false>
__device__ __forceinline__ void apply_tiles(ApplyStream<DEPTH, ROPE> &st, unsigned char *tileQ, int lane,
                                            const ApplyOperands<64, HILO> &A, float eps,
                                            const unsigned char *s_lds = nullptr, const float (*zf)[8] = nullptr)
{
    constexpr int NS = HILO ? 2 : 1;
    constexpr int KS = 4;
    constexpr int kRow = kRowBytes;
    constexpr int kTileBytes = kApplyTile * kRow;
    const int n = lane & 31, g = lane >> 5;
    const int wr_off = (lane >> 3) * kRow + (lane & 7) * 16;   // the lane's chunk of a coalesced tile

    auto round = [&](int i0) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            __builtin_amdgcn_sched_barrier(0);   // stages stay in program order (see state_accumulate)
            const bool valid = i0 + s < st.walk.count;
            const uint32_t out_off = st.walk.template offset<kApplyTile>(i0 + s, st.row_bytes);
            if (valid) {
                wave_lds_fence();
                st.rot.template begin_tile<kApplyTile>(st.walk, i0 + s);
                // the table lookups of the tile go out first; the ReLU and the plain tile fill their latency
                f32x2 cs[kApplyTile / 8][4];
#pragma unroll
                for (int j = 0; j < kApplyTile / 8; ++j) st.rot.fetch(s, j, cs[j]);
                u32x4 pq[kApplyTile / 8];
#pragma unroll
                for (int j = 0; j < kApplyTile / 8; ++j) {
                    pq[j] = relu_bf16x8(st.q[s][j]);                                   // phi(Q)
                    *reinterpret_cast<u32x4 *>(tileQ + wr_off + 8 * j * kRow) = pq[j];
                }
                if (ROPE) {
#pragma unroll
                    for (int j = 0; j < kApplyTile / 8; ++j)
                        *reinterpret_cast<u32x4 *>(tileQ + kTileBytes + wr_off + 8 * j * kRow) = st.rot.rotate_with(pq[j], cs[j]);
                }
            }
            st.request(s, i0 + s + DEPTH);   // refill this stage: DEPTH tiles ahead
            __builtin_amdgcn_sched_barrier(0);
            u32x4 o[kApplyTile / 8] = {};
            if (valid) {
                wave_lds_fence();
                f32x16 acc[2], accz;
                float den_valu = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) { acc[0][i] = 0.f; acc[1][i] = 0.f; accz[i] = 0.f; }
                if (DEN_VALU) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const u32x4 w = *reinterpret_cast<const u32x4 *>(tileQ + n * kRow + (16 * ks + 8 * g) * 2);
                        den_valu += bf16_lo(w.x) * zf[ks][0] + bf16_hi(w.x) * zf[ks][1] + bf16_lo(w.y) * zf[ks][2] +
                                    bf16_hi(w.y) * zf[ks][3] + bf16_lo(w.z) * zf[ks][4] + bf16_hi(w.z) * zf[ks][5] +
                                    bf16_lo(w.w) * zf[ks][6] + bf16_hi(w.w) * zf[ks][7];
                    }
                }
                // B operands: features 16*ks + 8g .. +8 of token n (br: the rotated copy for the numerator)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 bq = *reinterpret_cast<const bf16x8 *>(tileQ + n * kRow + (16 * ks + 8 * g) * 2);
                    const bf16x8 br = ROPE ? *reinterpret_cast<const bf16x8 *>(tileQ + kTileBytes + n * kRow +
                                                                               (16 * ks + 8 * g) * 2)
                                           : bq;
                    if (!DEN_VALU) accz = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.zrow[ks], bq, accz, 0, 0, 0);
#pragma unroll
                    for (int p = NS - 1; p >= 0; --p) {      // small (lo) terms first
                        const bf16x8 *sl = reinterpret_cast<const bf16x8 *>(s_lds);   // [hi/lo][row block][k-step][lane]
                        const bf16x8 a0 = S_LDS ? sl[((p * 2 + 0) * KS + ks) * 64 + lane] : A.s[p][0][ks];
                        const bf16x8 a1 = S_LDS ? sl[((p * 2 + 1) * KS + ks) * 64 + lane] : A.s[p][1][ks];
                        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, br, acc[0], 0, 0, 0);
                        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, br, acc[1], 0, 0, 0);
                    }
                }
                wave_lds_fence();
                // denominator: rows 0 (hi) and 1 (lo) of the z block sit in registers 0 and 1 of
                // the lanes of the lower half; the upper half fetches them across the wave
                float den;
                if (DEN_VALU) {
                    den = den_valu + __shfl_xor(den_valu, 32);   // the other half-wave holds the token's other 32 features
                } else {
                    den = accz[1] + accz[0];
                    den = __shfl(den, n);
                }
                const float inv = 1.0f / (den + eps);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    const f32x16 &a = acc[rb];
                    u32x4 lo4, hi4;
                    lo4.x = pack_bf16x2(a[0] * inv, a[1] * inv);
                    lo4.y = pack_bf16x2(a[2] * inv, a[3] * inv);
                    lo4.z = pack_bf16x2(a[4] * inv, a[5] * inv);
                    lo4.w = pack_bf16x2(a[6] * inv, a[7] * inv);
                    hi4.x = pack_bf16x2(a[8] * inv, a[9] * inv);
                    hi4.y = pack_bf16x2(a[10] * inv, a[11] * inv);
                    hi4.z = pack_bf16x2(a[12] * inv, a[13] * inv);
                    hi4.w = pack_bf16x2(a[14] * inv, a[15] * inv);
                    unsigned char *row = tileQ + n * kRow + (32 * g + 16 * rb) * 2;
                    *reinterpret_cast<u32x4 *>(row) = lo4;
                    *reinterpret_cast<u32x4 *>(row + 16) = hi4;
                }
                wave_lds_fence();
#pragma unroll
                for (int i = 0; i < kApplyTile / 8; ++i)
                    o[i] = *reinterpret_cast<const u32x4 *>(tileQ + wr_off + 8 * i * kRow);
            }
#pragma unroll
            for (int i = 0; i < kApplyTile / 8; ++i)
                store_stream16(st.rO, out_off + st.lane_off + (uint32_t)i * 8u * st.row_bytes, o[i]);
        }
    };
    // The first round stands apart so that the loop is entered with the same sequence of
    // outstanding loads and stores that its own rounds leave behind: the compiler sizes the
    // loop's waits for the worse of the two.
    if (st.walk.count > 0) round(0);
    for (int i0 = DEPTH; i0 < st.walk.count; i0 += DEPTH) round(i0);
}

// LDS bytes per wave and in total: one tile, two with ROPE (plain + rotated copy).
template <int ROPE>
__host__ __device__ constexpr int apply_wave_lds_bytes() { return (ROPE ? 2 : 1) * kApplyTile * kRowBytes; }
template <int WAVES, int ROPE>
__host__ __device__ constexpr int apply_lds_bytes() { return WAVES * apply_wave_lds_bytes<ROPE>(); }

// grid = (C, B*H), block = 64*WAVES.  Wave w of workgroup c owns tiles
// WAVES*c + w + WAVES*C*i (i = 0, 1, ...) of the T = ceil((t1-t0)/32) tiles,
// the same round-robin deal as the state kernel.  Without RoPE the host launches eight times as
// many workgroups as fit the device at once (four tiles per wave at 32 760 tokens and 32 heads):
// short-lived workgroups handed out in order by the dispatcher stream better than 256 that loop
// (pure copies show the same: 45 against 49 us), and what made them too expensive before - every
// wave fetching and converting all of S - is now done once per workgroup.
// HILO = false drops the low half of S (one MFMA pass instead of two).
// ROPE (kRopeNone/Table/3D); with kRope3D the dynamic LDS carries kRope3dLdsBytes more.
// S_LDS, DEN_VALU: the measurement variants of apply_tiles; S_LDS needs kApplyStateLdsBytes more dynamic LDS.
constexpr int kApplyStateLdsBytes = ApplyOperands<64, true>::kSharedBytes;
template <bool HILO, int WAVES, int DEPTH, int ROPE, bool S_LDS = false, bool DEN_VALU = false>
__global__ __launch_bounds__(64 * WAVES, 1) void apply_mfma_d64(
    const uint16_t *__restrict__ Q, uint16_t *__restrict__ O, RopeArg rope, TokStrides st, int H,
    int /* d: always 64; keeps the argument list of the d = 112/128 kernel */, int t0, int t1, int C, const float *__restrict__ S, const float *__restrict__ z, float eps)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const uint16_t *Qh = Q + b * st.b + h * st.h;
    uint16_t *Oh = O + b * st.b + h * st.h;
    const int n_tiles = (t1 - t0 + kApplyTile - 1) / kApplyTile;

    ApplyStream<DEPTH, ROPE> stream(Qh, Oh, rope, lds + apply_lds_bytes<WAVES, ROPE>(), st.n, t1, lane,
                                    TileWalk(t0, WAVES * c + wave, WAVES * C, n_tiles, bh));
    Rope3dFill tabs;
    if (ROPE == kRope3D) rope3d_lds_fill_begin(rope.r3, tabs);   // the first loads of the kernel
    apply_prefetch<0, DEPTH>(stream);   // in flight while S is fetched
    if (ROPE == kRope3D) {
        rope3d_lds_fill_end(lds + apply_lds_bytes<WAVES, ROPE>(), rope.r3, tabs);
        wg_barrier();
    }
    ApplyOperands<64, HILO> A;
    static_assert(apply_lds_bytes<WAVES, ROPE>() >= ApplyOperands<64, HILO>::kSharedBytes && WAVES == 4, "the tiles can stage S for load_shared");
    // through the tiles, not yet in use; S_LDS: into an area of their own behind the tiles (and the tables), to stay
    unsigned char *stage = S_LDS ? lds + apply_lds_bytes<WAVES, ROPE>() + (ROPE == kRope3D ? kRope3dLdsBytes : 0) : lds;
    A.template load_shared<false>(S + (size_t)bh * 64 * 64, z + (size_t)bh * 64, wave, lane, stage);
    float zf[4][8];
    if (DEN_VALU) load_key_sums<false>(z + (size_t)bh * 64, lane, zf);
    apply_tiles<HILO, DEPTH, ROPE, S_LDS, DEN_VALU>(stream, lds + wave * apply_wave_lds_bytes<ROPE>(), lane, A, eps, stage, zf);
}

}  // namespace sv
