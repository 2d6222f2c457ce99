// Token streaming for d = 112 and 128 (DP = 128): the waves of a workgroup work on the same tile
// together.
//
// With 64 features a wave can keep a whole 64 x 64 state (or a 64-column panel of it) to itself
// and never talks to its neighbours.  With 128 the state is four such quadrants and the apply
// needs several panels, so every token row is needed by more than one wave.  Letting all of them
// fetch it costs far more than the extra instructions: half rows of 224 or 256 bytes split cache
// lines between waves and the non-temporal streams fetch them twice (measured: 2.4 TB/s instead of
// 5.4).  Here each wave loads whole rows that nobody else loads, the tile is assembled in
// workgroup-shared LDS, and barriers hand it to the waves that compute:
//
//   state (the full-table RoPE form; the other forms use the wave-private kernel of
//          wide_state.hpp): wave w loads rows 8w .. 8w+8 of K and V of a 32-token tile, then
//          folds key block w%2 against value block w/2 (a 64 x 64 quadrant) from LDS; one barrier
//          per tile;
//   apply: wave w loads rows 8w .. 8w+8 of a 32-token Q tile, computes 32 of the 128 output
//          features of the whole tile (its 128 x 32 panel of S stays in registers) into a shared
//          output tile, then stores whole rows 8w .. 8w+8 of O; two barriers per tile, two
//          workgroups per compute unit (the stream and the loop are written for other splits of
//          the tile among the waves as well, see CoopApplyStream).
//
// Barriers are bare s_barrier instructions behind an LDS-only wait, so the global loads of later
// tiles and the stores of earlier ones stay in flight across them.  For d = 112 the features past
// 112 are addressed out of range: they read as zeros and their stores are dropped.
#pragma once

#include "apply_mfma.hpp"
#include "state_mfma.hpp"

namespace sv {

constexpr int kCoopRow = 128 * 2 + 16;           // LDS row: 128 bf16 features + padding
constexpr int kCoopTile = 32 * kCoopRow;         // one 32-token tile in LDS

// ---- state ---------------------------------------------------------------------------------------

// One wave's share of the workgroup's K/V stream: rows 8*wave .. +8 of every tile
// (16 lanes of 16 bytes per row, 4 rows per load instruction), DEPTH tiles in flight.
template <int DEPTH, int ROPE>
struct CoopStateStream {
    static constexpr int NLD = 2;
    rsrc_t rK, rV;
    uint32_t row_bytes, lane_off;
    bool valid;
    TileWalk walk;                       // the workgroup's tiles: identical in all four waves
    u32x4 k[DEPTH][NLD], v[DEPTH][NLD];
    Rotator<ROPE, NLD, DEPTH> rot;

    __device__ __forceinline__ CoopStateStream(const uint16_t *Kh, const uint16_t *Vh, const RopeArg &rope,
                                               const unsigned char *lds_tab, int64_t stride_n, int t1, int d, int wave,
                                               int lane, const TileWalk &w)
        : rK(make_rsrc(Kh, (uint32_t)t1 * (uint32_t)stride_n * 2u)),
          rV(make_rsrc(Vh, (uint32_t)t1 * (uint32_t)stride_n * 2u)), row_bytes((uint32_t)stride_n * 2u),
          lane_off((uint32_t)(8 * wave + (lane >> 4)) * (uint32_t)stride_n * 2u + (uint32_t)(lane & 15) * 16u),
          valid((lane & 15) * 8 < d), walk(w),
          rot(rope, t1, d, 8 * wave + (lane >> 4), 4, 4 * (lane & 15), 1, lds_tab) {}

    __device__ __forceinline__ void request(int s, int i)
    {
        const uint32_t base = valid ? walk.offset<32>(i, row_bytes) : kOutOfRange;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            k[s][j] = load_stream16(rK, base + lane_off + (uint32_t)j * 4u * row_bytes);
            v[s][j] = load_stream16(rV, base + lane_off + (uint32_t)j * 4u * row_bytes);
        }
        rot.request(s, i < walk.count, walk.token<32>(i));
    }
};

template <int DEPTH, int ROPE>
__device__ __forceinline__ void coop_state_prefetch(CoopStateStream<DEPTH, ROPE> &st)
{
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
        st.request(s, s);
        __builtin_amdgcn_sched_barrier(0);   // requests go out in stage order, as they do in the loop
    }
}

// LDS of the state phase: K and V tiles, double-buffered; with ROPE also the
// un-rotated phi(K) (the key sum is never rotated).
template <int ROPE> __host__ __device__ constexpr int coop_state_lds_bytes() { return (ROPE ? 6 : 4) * kCoopTile; }

// Accumulates quadrant (kb, vb) of the workgroup's partial state over the
// workgroup's tiles.  Must be called by all four waves (it contains barriers; the
// tile count is the same in all of them).  Key sums are kept by the waves with vb == 0.
//
// Software pipeline, one barrier per tile: while the matrix cores work on tile i
// (operands from LDS buffer i%2), the wave's vector ALU puts its rows of tile
// i+1 (ReLU, rotation) into the other buffer; the barrier at the end of the step
// says both that tile i+1 is complete and that everybody is done reading tile i,
// whose buffer the next step overwrites.
template <int DEPTH, int ROPE>
__device__ __forceinline__ void state_accumulate_coop(CoopStateStream<DEPTH, ROPE> &st, unsigned char *lds, int wave,
                                                      int lane, int kb, int vb, StateAcc &acc)
{
    static_assert(DEPTH % 2 == 0, "stage parity selects the LDS buffer");
    const int wr_off = (8 * wave + (lane >> 4)) * kCoopRow + (lane & 15) * 16;
    const uint32_t one2 = 0x3f803f80u;   // bf16 (1.0, 1.0)
    const u32x4 ones4 = {one2, one2, one2, one2};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones4);
    const int count = st.walk.count;
    if (count == 0) return;

    // This wave's rows of the workgroup's i-th tile go from stage s into LDS buffer s%2; the stage
    // is refilled DEPTH tiles ahead whether or not tile i exists (out of range nothing is read).
    auto prepare = [&](int s, int i) __attribute__((always_inline)) {
        unsigned char *bufK = lds + (s & 1) * kCoopTile, *bufV = lds + (2 + (s & 1)) * kCoopTile;
        unsigned char *bufP = lds + (4 + (s & 1)) * kCoopTile;   // un-rotated phi(K), ROPE only
        if (i < count) {
            st.rot.template begin_tile<32>(st.walk, i);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const u32x4 kk = relu_bf16x8(st.k[s][j]);
                if (ROPE) {
                    *reinterpret_cast<u32x4 *>(bufP + wr_off + 4 * j * kCoopRow) = kk;
                    *reinterpret_cast<u32x4 *>(bufK + wr_off + 4 * j * kCoopRow) = st.rot.rotate(s, j, kk);
                } else {
                    *reinterpret_cast<u32x4 *>(bufK + wr_off + 4 * j * kCoopRow) = kk;
                }
                *reinterpret_cast<u32x4 *>(bufV + wr_off + 4 * j * kCoopRow) = st.v[s][j];
            }
        }
        st.request(s, i + DEPTH);
    };

    prepare(0, 0);
    lds_barrier();
    for (int i0 = 0; i0 < count; i0 += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            __builtin_amdgcn_sched_barrier(0);   // stages stay in program order
            if (i0 + s < count) {
                const unsigned char *bufK = lds + (s & 1) * kCoopTile, *bufV = lds + (2 + (s & 1)) * kCoopTile;
                const unsigned char *bufP = ROPE ? lds + (4 + (s & 1)) * kCoopTile : bufK;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const bf16x8 a0 = lds_tr_operand<kCoopRow>(bufK, 16 * ks, 64 * kb, lane);
                    const bf16x8 a1 = lds_tr_operand<kCoopRow>(bufK, 16 * ks, 64 * kb + 32, lane);
                    const bf16x8 b0 = lds_tr_operand<kCoopRow>(bufV, 16 * ks, 64 * vb, lane);
                    const bf16x8 b1 = lds_tr_operand<kCoopRow>(bufV, 16 * ks, 64 * vb + 32, lane);
                    acc.s[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc.s[0][0], 0, 0, 0);
                    acc.s[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc.s[0][1], 0, 0, 0);
                    acc.s[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc.s[1][0], 0, 0, 0);
                    acc.s[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc.s[1][1], 0, 0, 0);
                    if (vb == 0) {
                        const bf16x8 p0 = ROPE ? lds_tr_operand<kCoopRow>(bufP, 16 * ks, 64 * kb, lane) : a0;
                        const bf16x8 p1 = ROPE ? lds_tr_operand<kCoopRow>(bufP, 16 * ks, 64 * kb + 32, lane) : a1;
                        acc.zm[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p0, ones, acc.zm[0], 0, 0, 0);
                        acc.zm[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1, ones, acc.zm[1], 0, 0, 0);
                    }
                }
            }
            prepare((s + 1) % DEPTH, i0 + s + 1);
            __builtin_amdgcn_sched_barrier(0);
            if (i0 + s < count) lds_barrier();
        }
    }
}

// ---- apply ---------------------------------------------------------------------------------------

// One wave's share of the workgroup's Q/O stream, both for the loads of Q and for the stores of O.
// A wave computes NB blocks of 32 output features, so 4/NB waves work on one 32-token tile and a
// workgroup of WAVES waves takes WAVES*NB/4 tiles per step; its rows are dealt evenly to the waves:
//   WAVES = 4, NB = 1   one tile, 8 rows per wave, few enough registers for two waves per SIMD (in use)
//   WAVES = 4, NB = 2   a pair of tiles per step, 16 rows per wave
//   WAVES = 2, NB = 2   one tile, 16 rows per wave
template <int DEPTH, int ROPE, int WAVES, int NB>
struct CoopApplyStream {
    static constexpr int STEP = 8 * WAVES * NB;   // tokens per workgroup step
    static constexpr int ROWS = STEP / WAVES;     // rows per wave
    static constexpr int NLD = ROWS / 4;          // 4 rows per load instruction
    rsrc_t rQ, rO;
    uint32_t row_bytes, lane_off;
    bool valid;
    TileWalk walk;                       // the workgroup's steps (units of STEP tokens)
    u32x4 q[DEPTH][NLD];
    Rotator<ROPE, NLD, DEPTH> rot;

    __device__ __forceinline__ CoopApplyStream(const uint16_t *Qh, uint16_t *Oh, const RopeArg &rope,
                                               const unsigned char *lds_tab, int64_t stride_n, int t1, int d, int wave,
                                               int lane, const TileWalk &w)
        : rQ(make_rsrc(Qh, (uint32_t)t1 * (uint32_t)stride_n * 2u)),
          rO(make_rsrc(Oh, (uint32_t)t1 * (uint32_t)stride_n * 2u)), row_bytes((uint32_t)stride_n * 2u),
          lane_off((uint32_t)(ROWS * wave + (lane >> 4)) * (uint32_t)stride_n * 2u + (uint32_t)(lane & 15) * 16u),
          valid((lane & 15) * 8 < d), walk(w),
          rot(rope, t1, d, ROWS * wave + (lane >> 4), 4, 4 * (lane & 15), 1, lds_tab) {}

    __device__ __forceinline__ void request(int s, int i)
    {
        const uint32_t base = valid ? walk.offset<STEP>(i, row_bytes) : kOutOfRange;
#pragma unroll
        for (int j = 0; j < NLD; ++j) q[s][j] = load_stream16(rQ, base + lane_off + (uint32_t)j * 4u * row_bytes);
        rot.request(s, i < walk.count, walk.token<STEP>(i));
    }
};

template <int FROM, int TO, int DEPTH, int ROPE, int WAVES, int NB>
__device__ __forceinline__ void coop_apply_prefetch(CoopApplyStream<DEPTH, ROPE, WAVES, NB> &st)
{
#pragma unroll
    for (int s = FROM; s < TO; ++s) {
        st.request(s, s);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// LDS of the apply phase: the Q tiles of a step (as the MFMAs want them: rotated with ROPE), its
// O tiles and the denominators of its tokens.
template <int WAVES, int NB> __host__ __device__ constexpr int coop_apply_lds_bytes() {
    return 2 * (WAVES * NB / 4) * kCoopTile + 8 * WAVES * NB * 4;
}

// Applies the state panel in `A` (value block wave % (4/NB)) to tile wave / (4/NB) of every step
// of the workgroup's share.  Must be called by all waves of the workgroup.
//
// Denominators phi(Q_i) . z + eps: the wave that loads a row also takes its dot product with z on
// the vector ALU (a lane holds eight features of the row and the matching eight of z, `zr`; 16
// lanes share a row) and leaves it in LDS beside the tile.  The products are exact in fp32, the
// unrotated phi(Q) is at hand there even with ROPE, and the matrix core is left with the numerator.
template <bool HILO, int DEPTH, int ROPE, int WAVES, int NB>
__device__ __forceinline__ void apply_tiles_coop(CoopApplyStream<DEPTH, ROPE, WAVES, NB> &st, unsigned char *lds,
                                                 int wave, int lane, const ApplyOperands<128, HILO, NB, false> &A,
                                                 const float (&zr)[8], float eps)
{
    constexpr int NS = HILO ? 2 : 1;
    constexpr int STEP = 8 * WAVES * NB, TILES = WAVES * NB / 4, ROWS = STEP / WAVES, NLD = ROWS / 4, WT = 4 / NB;
    const int t = wave / WT, vb = wave % WT;
    const int n = lane & 31, g = lane >> 5;
    unsigned char *bufQ = lds, *bufO = lds + TILES * kCoopTile;
    float *den = reinterpret_cast<float *>(lds + 2 * TILES * kCoopTile);            // [STEP]
    const int my_row = ROWS * wave + (lane >> 4);                                   // + 4 j: the rows this lane loads
    const int wr_off = my_row * kCoopRow + (lane & 15) * 16;
    const unsigned char *brow = bufQ + (32 * t + n) * kCoopRow;
    unsigned char *orow = bufO + (32 * t + n) * kCoopRow + (32 * NB * vb + 16 * NB * g) * 2;

    auto round = [&](int i0) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            __builtin_amdgcn_sched_barrier(0);   // stages stay in program order
            const bool valid = i0 + s < st.walk.count;
            const uint32_t out_off = st.valid ? st.walk.template offset<STEP>(i0 + s, st.row_bytes) : kOutOfRange;
            if (valid) {
                st.rot.template begin_tile<STEP>(st.walk, i0 + s);
                // the table lookups of the step go out first; ReLU and denominators fill their latency
                f32x2 cs[NLD][4];
#pragma unroll
                for (int j = 0; j < NLD; ++j) st.rot.fetch(s, j, cs[j]);
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    const u32x4 pq = relu_bf16x8(st.q[s][j]);                          // phi(Q)
                    float dot = bf16_lo(pq.x) * zr[0];
                    dot = __builtin_fmaf(bf16_hi(pq.x), zr[1], dot);
                    dot = __builtin_fmaf(bf16_lo(pq.y), zr[2], dot);
                    dot = __builtin_fmaf(bf16_hi(pq.y), zr[3], dot);
                    dot = __builtin_fmaf(bf16_lo(pq.z), zr[4], dot);
                    dot = __builtin_fmaf(bf16_hi(pq.z), zr[5], dot);
                    dot = __builtin_fmaf(bf16_lo(pq.w), zr[6], dot);
                    dot = __builtin_fmaf(bf16_hi(pq.w), zr[7], dot);
                    dot += __shfl_xor(dot, 1);                                          // the 16 lanes of the row
                    dot += __shfl_xor(dot, 2);
                    dot += __shfl_xor(dot, 4);
                    dot += __shfl_xor(dot, 8);
                    if ((lane & 15) == 0) den[my_row + 4 * j] = dot;
                    *reinterpret_cast<u32x4 *>(bufQ + wr_off + 4 * j * kCoopRow) = st.rot.rotate_with(pq, cs[j]);
                }
            }
            st.request(s, i0 + s + DEPTH);   // refill this stage: DEPTH steps ahead
            __builtin_amdgcn_sched_barrier(0);
            u32x4 o[NLD] = {};
            if (valid) {
                // Q tiles and denominators complete.  They are overwritten in the next round, by waves
                // that have passed the second barrier below, which every wave reaches after its reads.
                lds_barrier();
                f32x16 acc[NB];
#pragma unroll
                for (int i = 0; i < 16; ++i)
#pragma unroll
                    for (int rb = 0; rb < NB; ++rb) acc[rb][i] = 0.f;
                const float inv = 1.0f / (den[32 * t + n] + eps);
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const bf16x8 bq = *reinterpret_cast<const bf16x8 *>(brow + (16 * ks + 8 * g) * 2);
#pragma unroll
                    for (int p = NS - 1; p >= 0; --p) {      // small (lo) terms first
#pragma unroll
                        for (int rb = 0; rb < NB; ++rb)
                            acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.s[p][rb][ks], bq, acc[rb], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int rb = 0; rb < NB; ++rb) {
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
                    *reinterpret_cast<u32x4 *>(orow + 32 * rb) = lo4;
                    *reinterpret_cast<u32x4 *>(orow + 32 * rb + 16) = hi4;
                }
                // O tiles complete after this barrier; they are overwritten after the first
                // barrier of the next round, which every wave reaches after the reads below.
                lds_barrier();
#pragma unroll
                for (int j = 0; j < NLD; ++j) o[j] = *reinterpret_cast<const u32x4 *>(bufO + wr_off + 4 * j * kCoopRow);
            }
#pragma unroll
            for (int j = 0; j < NLD; ++j)
                store_stream16(st.rO, out_off + st.lane_off + (uint32_t)j * 4u * st.row_bytes, o[j]);
        }
    };
    // first round apart: the loop is entered in its own steady state of outstanding loads and stores
    if (st.walk.count > 0) round(0);
    for (int i0 = DEPTH; i0 < st.walk.count; i0 += DEPTH) round(i0);
}

// ---- kernels ---------------------------------------------------------------------------------------

// Dynamic LDS: the larger of the streaming buffers and the four reduction slots.
template <int ROPE>
__host__ __device__ constexpr int state_d128_lds_bytes() {
    return (coop_state_lds_bytes<ROPE>() > 4 * kStateElems * 4 ? coop_state_lds_bytes<ROPE>() : 4 * kStateElems * 4) +
           kEpochLdsBytes;
}

// State reduction for d = 112 or 128.  grid = (C, B*H), block = 256; workgroup c
// owns tiles c + C*i of the T = ceil((t1-t0)/32) tiles.  FINALIZE and ROPE as in
// state_mfma_d64; partial states and S are d x d with row length d.
template <int DEPTH, bool FINALIZE, int ROPE>
__global__ __launch_bounds__(256, 1) void state_mfma_d128(
    const uint16_t *__restrict__ K, const uint16_t *__restrict__ V, RopeArg rope, TokStrides st,
    int H, int d, int t0, int t1, int C, const float *S_in, const float *z_in, float *S_out, float *z_out,
    void *__restrict__ ws, unsigned long long epoch, uint32_t spin_limit)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x, bh = blockIdx.y, BH = gridDim.y;
    const int b = bh / H, h = bh % H;
    const int elems = d * d + d;
    const uint16_t *Kh = K + b * st.b + h * st.h;
    const uint16_t *Vh = V + b * st.b + h * st.h;
    const int n_tiles = (t1 - t0 + 31) / 32;
    EpochSource es;
    if (FINALIZE) es.begin(ws, BH, elems, epoch, bh, c, C);

    StateAcc acc;
    acc.clear();
    CoopStateStream<DEPTH, ROPE> stream(Kh, Vh, rope, lds + state_d128_lds_bytes<ROPE>(), st.n, t1, d, wave, lane,
                                        TileWalk(t0, c, C, n_tiles, bh));
    Rope3dFill tabs;
    if (ROPE == kRope3D) rope3d_lds_fill_begin(rope.r3, tabs);   // the first loads of the kernel
    coop_state_prefetch(stream);
    if (ROPE == kRope3D) {
        rope3d_lds_fill_end(lds + state_d128_lds_bytes<ROPE>(), rope.r3, tabs);
        wg_barrier();
    }
    state_accumulate_coop(stream, lds, wave, lane, wave & 1, wave >> 1, acc);

    float *partials = static_cast<float *>(ws) + (size_t)bh * kMaxChunks * elems;
    state_wg_quadrant_store(acc, reinterpret_cast<float *>(lds), wave, lane, d, partials + (size_t)c * elems);
    if (FINALIZE) {
        epoch = es.resolve(reinterpret_cast<unsigned long long *>(lds + state_d128_lds_bytes<ROPE>() - kEpochLdsBytes));
        const float *Sc = S_in ? S_in + (size_t)bh * d * d : nullptr, *zc = z_in + (size_t)bh * d;
        const StateSlice sl(c, C, d);
        f32x2 carry[3];
        state_slice_carry<256>(sl, Sc, zc, (int)threadIdx.x, carry);
        if (!state_publish_and_wait(ws, BH, elems, bh, c, C, 0, epoch, spin_limit, lane))
            return;                                     // timed out: this wave leaves its part of S, z as it was
        state_finalize_slice<256, false>(partials, sl, C, Sc, zc, S_out + (size_t)bh * d * d, z_out + (size_t)bh * d,
                                         (int)threadIdx.x, carry);
    }
}

// Apply for d = 112 or 128.  grid = (C, B*H), block = 64 * WAVES; workgroup c owns the steps
// c + C*i of the ceil((t1-t0)/STEP) steps of STEP = 8*WAVES*NB tokens (see CoopApplyStream).
// With NB = 1 a wave keeps one 128 x 32 panel of S and fits in half a SIMD's registers: two
// workgroups (eight waves) share a compute unit, and while one wave waits at a barrier or works on
// the vector ALU (ReLU, rotation, scaling) the other wave of its SIMD feeds the matrix core.
template <bool HILO, int DEPTH, int ROPE, int WAVES, int NB>
__global__ __launch_bounds__(64 * WAVES, NB == 1 ? 2 : 1) void apply_mfma_d128(
    const uint16_t *__restrict__ Q, uint16_t *__restrict__ O, RopeArg rope, TokStrides st, int H,
    int d, int t0, int t1, int C, const float *__restrict__ S, const float *__restrict__ z, float eps)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x, bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const uint16_t *Qh = Q + b * st.b + h * st.h;
    uint16_t *Oh = O + b * st.b + h * st.h;
    constexpr int STEP = 8 * WAVES * NB;
    const int n_steps = (t1 - t0 + STEP - 1) / STEP;

    CoopApplyStream<DEPTH, ROPE, WAVES, NB> stream(Qh, Oh, rope, lds + coop_apply_lds_bytes<WAVES, NB>(), st.n, t1,
                                                   d, wave, lane, TileWalk(t0, c, C, n_steps, bh));
    Rope3dFill tabs;
    if (ROPE == kRope3D) rope3d_lds_fill_begin(rope.r3, tabs);   // the first loads of the kernel
    coop_apply_prefetch<0, DEPTH>(stream);   // in flight while S is fetched
    if (ROPE == kRope3D) {
        rope3d_lds_fill_end(lds + coop_apply_lds_bytes<WAVES, NB>(), rope.r3, tabs);
        wg_barrier();
    }
    ApplyOperands<128, HILO, NB, false> A;
    A.template load<false>(S + (size_t)bh * d * d, z + (size_t)bh * d, d, wave % (4 / NB), lane);
    float zr[8];                                   // the key sums of the eight features this lane loads of a row
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int k = 8 * (lane & 15) + e;
        const float x = z[(size_t)bh * d + (k < d ? k : 0)];   // loaded by every lane: a load under a condition is a branch
        zr[e] = k < d ? x : 0.f;
    }
    apply_tiles_coop<HILO>(stream, lds, wave, lane, A, zr, eps);
}

}  // namespace sv
