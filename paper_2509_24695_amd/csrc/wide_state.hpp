// State reduction for d = 112 and 128 with wave-private tiles (no workgroup barrier in the token loop).
//
//   S[k][v] (+)= sum_j phi(K[j][k]) V[j][v],   z[k] (+)= sum_j phi(K[j][k])
//
// (brackets of the linear-attention equation of Sec. 3.2; with ROPE the keys that meet V are
// rotated after the ReLU, the key sum is not).
//
// The design of the d = 64 kernel carried over to a 128 x 128 state: every wave works alone on
// tiles of 16 tokens (one MFMA k-step) and holds the whole partial state, sixteen 32 x 32
// accumulators = 256 registers, which is what one wave per SIMD can afford.  Loads are whole
// 256-byte rows (16 lanes of 16 bytes, 4 rows per instruction), the tile goes through the wave's
// own LDS, transposing LDS reads deliver four key and four value operands, 16 MFMAs per tile.
// The key sum is kept per lane on the vector ALU (a lane always loads the same eight features).
// Compared with the workgroup-cooperative kernel (one 32-token tile shared by the four waves
// behind a barrier) the per-tile costs that do not shrink with the tile - position arithmetic of
// the rotation, waits, the barrier itself - are paid per 64 tokens of a compute unit's work
// instead of per 32 and never hold up the other waves.
//
// At the end the four waves' states are added in a fixed order, exchanged through LDS in the
// accumulators' own layout, and stored as the workgroup's partial.
#pragma once

#include "state_mfma.hpp"

namespace sv {

constexpr int kWideTile = 16;                       // tokens per tile: one MFMA k-step
// LDS row: 128 bf16 features + padding.  A transposing read takes 64 contiguous bytes from each of
// four consecutive rows per half wave; with a row pitch of 80 words the four 16-bank windows tile
// the 64 banks (a pitch of 68 words, enough for 16-byte reads, made them overlap: 44 % of the LDS
// cycles of this kernel were bank conflicts).
constexpr int kWideRow = 128 * 2 + 64;
constexpr int kWideTileBytes = kWideTile * kWideRow;

// LDS map (bytes): the K/V tiles (8 tiles from 0) and, from 64 KB, the rotation tables; once the token
// loop is over, [0, 128 KB) are the four waves' parcels of the final reduction; then the waves' key
// sums and the epoch word.
constexpr int kWideTabOffset = 64 * 1024;
constexpr int kWideParcelBytes = 8 * 16 * kWave * 4;     // eight accumulator blocks
constexpr int kWideZOffset = 4 * kWideParcelBytes;
constexpr int kWideEpochOffset = kWideZOffset + 4 * 128 * 4;
constexpr int kWideLdsBytes = kWideEpochOffset + kEpochLdsBytes;
static_assert(8 * kWideTileBytes <= kWideTabOffset, "the tiles end where the tables begin");
static_assert(kWideTabOffset + kRope3dLdsBytes <= kWideZOffset, "the tables end where the key sums begin");

struct WideAcc {
    // [r][value feature block]; in wave w, r is key feature block r ^ w: the final reduction then sends
    // and keeps the same registers in every wave
    f32x16 s[4][4];
    float z[8];       // features 8 * (lane % 16) + e of the tokens this lane loaded
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[rb][cb][i] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = 0.f;
    }
};

// One wave's input stream: rows lane/16 + 4 j of every tile of its walk, DEPTH tiles in flight.
// Lanes whose features lie past d (d = 112) address out of range: they read zeros.
template <int DEPTH, int ROPE>
struct WideStateStream {
    static constexpr int NLD = kWideTile / 4;
    rsrc_t rK, rV;
    uint32_t row_bytes, lane_off;
    bool valid;
    TileWalk walk;
    u32x4 k[DEPTH][NLD], v[DEPTH][NLD];
    Rotator<ROPE, NLD, DEPTH> rot;

    __device__ __forceinline__ WideStateStream(const uint16_t *Kh, const uint16_t *Vh, const RopeArg &rope,
                                               const unsigned char *lds_tab, int64_t stride_n, int t1, int d, int lane,
                                               const TileWalk &w)
        : rK(make_rsrc(Kh, (uint32_t)t1 * (uint32_t)stride_n * 2u)),
          rV(make_rsrc(Vh, (uint32_t)t1 * (uint32_t)stride_n * 2u)), row_bytes((uint32_t)stride_n * 2u),
          lane_off((uint32_t)(lane >> 4) * (uint32_t)stride_n * 2u + (uint32_t)(lane & 15) * 16u),
          valid((lane & 15) * 8 < d), walk(w), rot(rope, t1, d, lane >> 4, 4, 4 * (lane & 15), 1, lds_tab) {}

    __device__ __forceinline__ void request(int s, int i)
    {
        const uint32_t base = valid ? walk.offset<kWideTile>(i, row_bytes) : kOutOfRange;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            k[s][j] = load_stream16(rK, base + lane_off + (uint32_t)j * 4u * row_bytes);
            v[s][j] = load_stream16(rV, base + lane_off + (uint32_t)j * 4u * row_bytes);
        }
        rot.request(s, i < walk.count, walk.token<kWideTile>(i));
    }
};

template <int DEPTH, int ROPE>
__device__ __forceinline__ void wide_state_prefetch(WideStateStream<DEPTH, ROPE> &st)
{
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
        st.request(s, s);
        __builtin_amdgcn_sched_barrier(0);   // requests go out in stage order, as they do in the loop
    }
}

// ReLU, key sums and rotation of the tile in stage s, in the registers it was loaded into; the
// rotator has been told the tile (begin_tile).  Straight-line code, so that it can share a
// scheduling region with MFMAs.  Two chunks at a time: their eight table lookups go out first,
// ReLU and key sums fill the latency.
template <int DEPTH, int ROPE>
__device__ __forceinline__ void wide_state_prepare(WideStateStream<DEPTH, ROPE> &st, int s, WideAcc &acc)
{
    constexpr int NLD = WideStateStream<DEPTH, ROPE>::NLD;
#pragma unroll
    for (int j0 = 0; j0 < NLD; j0 += 2) {
        f32x2 cs[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) st.rot.fetch(s, j0 + j, cs[j]);
#pragma unroll
        for (int j = j0; j < j0 + 2; ++j) {
            const u32x4 kk = relu_bf16x8(st.k[s][j]);
            acc.z[0] += bf16_lo(kk.x);  acc.z[1] += bf16_hi(kk.x);
            acc.z[2] += bf16_lo(kk.y);  acc.z[3] += bf16_hi(kk.y);
            acc.z[4] += bf16_lo(kk.z);  acc.z[5] += bf16_hi(kk.z);
            acc.z[6] += bf16_lo(kk.w);  acc.z[7] += bf16_hi(kk.w);
            st.k[s][j] = kk;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) st.k[s][j0 + j] = st.rot.rotate_with(st.k[s][j0 + j], cs[j]);
    }
}

// Accumulates the wave's share (its first DEPTH tiles are requested).  Stages past the share and
// tokens past t1 hold zeros and add nothing.  tileK, tileV: the wave's private LDS tiles.
// Software-pipelined by one tile: with one wave per SIMD nothing else fills the matrix core's
// shadow, so the vector work of tile i + 1 is issued between the MFMAs of tile i.
template <int DEPTH, int ROPE>
__device__ __forceinline__ void wide_state_accumulate(WideStateStream<DEPTH, ROPE> &st, unsigned char *tileK,
                                                      unsigned char *tileV, int wave, int lane, WideAcc &acc)
{
    constexpr int NLD = WideStateStream<DEPTH, ROPE>::NLD;
    const int wr_off = (lane >> 4) * kWideRow + (lane & 15) * 16;
    st.rot.template begin_tile<kWideTile>(st.walk, 0);
    wide_state_prepare(st, 0, acc);
    for (int i0 = 0; i0 < st.walk.count; i0 += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            __builtin_amdgcn_sched_barrier(0);   // stages stay in program order
            wave_lds_fence();   // earlier reads of the tile buffers are done before they are overwritten
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                *reinterpret_cast<u32x4 *>(tileK + wr_off + 4 * j * kWideRow) = st.k[s][j];
                *reinterpret_cast<u32x4 *>(tileV + wr_off + 4 * j * kWideRow) = st.v[s][j];
            }
            st.request(s, i0 + s + DEPTH);   // refill this stage: DEPTH tiles ahead
            __builtin_amdgcn_sched_barrier(0);
            // the next tile's position (has branches: kept out of the MFMA region)
            st.rot.template begin_tile<kWideTile>(st.walk, i0 + s + 1);
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_fence();
            bf16x8 a[4], b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a[q] = lds_tr_operand<kWideRow>(tileK, 0, 32 * (q ^ wave), lane);
                b[q] = lds_tr_operand<kWideRow>(tileV, 0, 32 * q, lane);
            }
            __builtin_amdgcn_sched_barrier(0);
            wide_state_prepare(st, (s + 1) % DEPTH, acc);
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc.s[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rb], b[cb], acc.s[rb][cb], 0, 0, 0);
            // one MFMA, then a share of the other instructions, sixteen times over
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x106, ROPE == kRopeNone ? 6 : 17, 0);
            }
        }
    }
}

// Accumulator blocks travel between waves through LDS as each lane's own registers: block `slot` of a
// transfer is four 16-byte words per lane, lane-contiguous (1 KB per instruction, no bank conflicts),
// and the partner's lane of the same number holds the same elements of S.
__device__ __forceinline__ void wide_send(unsigned char *region, int slot, const f32x16 &a, int lane)
{
    f32x4 *p = reinterpret_cast<f32x4 *>(region) + slot * 4 * kWave + lane;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f32x4 x;
        x.x = a[4 * q];  x.y = a[4 * q + 1];  x.z = a[4 * q + 2];  x.w = a[4 * q + 3];
        p[q * kWave] = x;
    }
}
// out(b) = own(b) + block b of the parcel at `region`, b < N.  The LDS reads run one block ahead of
// the additions and no further: left to itself the compiler requests the whole parcel at once and
// spills the state to make room for it.
template <int N, class OwnFn, class OutFn>
__device__ __forceinline__ void wide_recv_add(const unsigned char *region, int lane, OwnFn own, OutFn out)
{
    const f32x4 *p = reinterpret_cast<const f32x4 *>(region) + lane;
    f32x4 x[2][4];
#pragma unroll
    for (int q = 0; q < 4; ++q) x[0][q] = p[q * kWave];
#pragma unroll
    for (int b = 0; b < N; ++b) {
        if (b + 1 < N) {
#pragma unroll
            for (int q = 0; q < 4; ++q) x[(b + 1) & 1][q] = p[((b + 1) * 4 + q) * kWave];
        }
        __builtin_amdgcn_sched_barrier(0);
        const f32x16 &o = own(b);
        f32x16 r;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 y = x[b & 1][q];
            r[4 * q] = o[4 * q] + y.x;          r[4 * q + 1] = o[4 * q + 1] + y.y;
            r[4 * q + 2] = o[4 * q + 2] + y.z;  r[4 * q + 3] = o[4 * q + 3] + y.w;
        }
        out(b) = r;
        __builtin_amdgcn_sched_barrier(0);
    }
}
// Adds the four waves' states in the fixed order (w0 + w2) + (w1 + w3) and stores the workgroup's
// partial (d x d, row length d, then the d key sums) to `out` with coherent stores.  Must be called
// by all threads; the tiles and tables in LDS are dead afterwards.
//
// Two exchanges in the registers' own layout, each halving what a wave still owns: waves w and w ^ 2
// swap the halves of S the other one keeps (32 KB each way) and add, then w and w ^ 1 swap one band
// of 32 key features (16 KB).  Wave w ends with band w of the sum and stores it straight from its
// accumulators, 32 consecutive floats of two rows per instruction.  Because block r of wave w holds
// key block r ^ w (see WideAcc), the blocks that go out are blocks 2, 3 and then block 1 in every
// wave, and a parcel's block meets the same key features at the receiver: one code path, whose only
// dependence on the wave is in addresses.  192 KB go through LDS in 16-byte words; laying all four
// states out row-major and re-reading them (256 KB of 4-byte writes, which move 64 bytes a clock, and
// as much again in reads) took 4.8 us of a 22 us kernel.
// A wave's second parcel goes where it read its first (nobody else touches that region any more),
// so the exchanges need one barrier each.
__device__ __forceinline__ void wide_state_wg_reduce_store(WideAcc &acc, unsigned char *lds, int wave, int lane, int d,
                                                           float *__restrict__ out)
{
    float *zs = reinterpret_cast<float *>(lds + kWideZOffset);  // [wave][128]
    // key sums: lanes with equal lane % 16 hold the same eight features
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float x = acc.z[e];
        x += __shfl_xor(x, 16);
        x += __shfl_xor(x, 32);
        acc.z[e] = x;
    }
    wg_barrier();                                   // all waves are done with their tiles
    if (lane < 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) zs[wave * 128 + lane * 8 + e] = acc.z[e];
    }
    unsigned char *mine = lds + wave * kWideParcelBytes, *theirs = lds + (wave ^ 2) * kWideParcelBytes;
    const unsigned char *from = lds + (wave ^ 3) * kWideParcelBytes;   // where wave ^ 1 read its first parcel
    // with wave ^ 2: blocks 2, 3 go out; what comes in belongs to blocks 0, 1
#pragma unroll
    for (int rr = 0; rr < 2; ++rr)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) wide_send(mine, 4 * rr + cb, acc.s[2 + rr][cb], lane);
    lds_barrier();                                  // LDS only
    f32x16 h[2][4], fin[4];
    wide_recv_add<8>(theirs, lane, [&](int b) -> const f32x16 & { return acc.s[b >> 2][b & 3]; },
                     [&](int b) -> f32x16 & { return h[b >> 2][b & 3]; });
    // with wave ^ 1: block 1 goes out (`theirs` is this wave's to overwrite now), block 0 is band `wave`
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) wide_send(theirs, cb, h[1][cb], lane);
    lds_barrier();
    wide_recv_add<4>(from, lane, [&](int b) -> const f32x16 & { return h[0][b]; },
                     [&](int b) -> f32x16 & { return fin[b]; });
    // element i of block cb: row 32 wave + 8 (i / 4) + 4 (lane / 32) + i % 4, column 32 cb + lane % 32.
    // Rows past d lie past the resource's end, columns past d are sent there: both are dropped.
    const int n = lane & 31, g = lane >> 5;
    const rsrc_t rS = make_rsrc(out, (uint32_t)d * (uint32_t)d * 4u);
    const uint32_t base = ((uint32_t)(32 * wave + 4 * g) * (uint32_t)d + (uint32_t)n) * 4u;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const uint32_t col = 32 * cb + n < d ? base + 128u * cb : kOutOfRange;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            store_coherent4(rS, col + (uint32_t)(8 * (i >> 2) + (i & 3)) * (uint32_t)d * 4u, fin[cb][i]);
    }
    const int half = d / 2;
    for (int u = threadIdx.x; u < half; u += 4 * kWave) {
        const int k = 2 * u;
        f32x2 x;
        x.x = (zs[k] + zs[256 + k]) + (zs[128 + k] + zs[384 + k]);
        x.y = (zs[k + 1] + zs[256 + k + 1]) + (zs[128 + k + 1] + zs[384 + k + 1]);
        store_coherent(out + (size_t)d * d + k, x);
    }
}

// grid = (C, B*H), block = 256.  Wave w of workgroup c owns tiles 4c + w + 4C i of the
// T = ceil((t1 - t0) / 16) tiles.  FINALIZE as in state_mfma_d64.  ROPE: kRopeNone or kRope3D (the
// table rows of kRopeTable do not fit in the registers left beside the state).
template <int DEPTH, bool FINALIZE, int ROPE>
__global__ __launch_bounds__(256, 1) void state_mfma_wide(
    const uint16_t *__restrict__ K, const uint16_t *__restrict__ V, RopeArg rope, TokStrides st,
    int H, int d, int t0, int t1, int C, const float *S_in, const float *z_in, float *S_out, float *z_out,
    void *__restrict__ ws, unsigned long long epoch, uint32_t spin_limit)
{
    static_assert(ROPE == kRopeNone || ROPE == kRope3D, "no full-table form of this kernel");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x, bh = blockIdx.y, BH = gridDim.y;
    const int b = bh / H, h = bh % H;
    const int elems = d * d + d;
    const uint16_t *Kh = K + b * st.b + h * st.h;
    const uint16_t *Vh = V + b * st.b + h * st.h;
    const int n_tiles = (t1 - t0 + kWideTile - 1) / kWideTile;
    EpochSource es;
    if (FINALIZE) es.begin(ws, BH, elems, epoch, bh, c, C);

    WideAcc acc;
    acc.clear();
    WideStateStream<DEPTH, ROPE> stream(Kh, Vh, rope, lds + kWideTabOffset, st.n, t1, d, lane,
                                        TileWalk(t0, 4 * c + wave, 4 * C, n_tiles, bh));
    Rope3dFill tabs;
    if (ROPE == kRope3D) rope3d_lds_fill_begin(rope.r3, tabs);   // the first loads of the kernel
    wide_state_prefetch(stream);
    if (ROPE == kRope3D) {
        rope3d_lds_fill_end(lds + kWideTabOffset, rope.r3, tabs);
        wg_barrier();
    }
    unsigned char *tileK = lds + wave * 2 * kWideTileBytes, *tileV = tileK + kWideTileBytes;
    wide_state_accumulate(stream, tileK, tileV, wave, lane, acc);

    float *partials = static_cast<float *>(ws) + (size_t)bh * kMaxChunks * elems;
    wide_state_wg_reduce_store(acc, lds, wave, lane, d, partials + (size_t)c * elems);
    if (FINALIZE) {
        epoch = es.resolve(reinterpret_cast<unsigned long long *>(lds + kWideEpochOffset));
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

}  // namespace sv
