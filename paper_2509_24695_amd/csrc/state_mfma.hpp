// bf16 MFMA state reduction for d = 64 on gfx950 (and the parts shared with d = 112, 128).
//
//   S[k][v] (+)= sum_j phi(K[j][k]) V[j][v],   z[k] (+)= sum_j phi(K[j][k])
//
// (numerator and denominator brackets of the linear-attention equation of
// Sec. 3.2; the per-token states S_j of Sec. 3.3.1 summed over a token range).
//
// The contraction runs over tokens, but K and V are stored feature-contiguous,
// so both MFMA operands need a transpose.  Each wave works alone on tiles of
// TILE tokens: coalesced non-temporal 16-byte loads (8 lanes cover 128 bytes of
// a token row), ReLU on the packed bf16 pairs, a store into the wave's private
// LDS tile, and transposing LDS reads (ds_read_b64_tr_b16: 16 lanes fetch four
// 32-byte row segments and each lane receives its column of them, i.e. one
// feature of four consecutive tokens) that deliver the operands ready-made.
// The key sum comes out of the same pass as a product with a block of ones
// (exact: phi(K) times 1.0, fp32 accumulation).  Because a wave only ever reads
// LDS it wrote itself, no workgroup barrier is needed inside the token loop.
//
// One workgroup per compute unit and a round-robin deal of tiles keep the whole
// grid streaming through a narrow, moving window of each head's tokens, which
// is what HBM likes best; the loads of the next DEPTH tiles are always in
// flight.  Workgroup partials go to the workspace; once all partials of a head
// are published, each of its workgroups adds up one slice of them in chunk
// order (bit-reproducible, no float atomics).
//
// d = 112 and 128 are served by the workgroup-cooperative kernels of coop128.hpp,
// which reuse the pieces below (tile walk, transposing reads, accumulators,
// partial-state reduction).
#pragma once

#include "common.hpp"
#include "rope.hpp"
#include "sync.hpp"

namespace sv {

constexpr int kRowBytes = 144;   // 128-byte token row + 16 bytes of padding (bank spread, keeps 16-byte alignment)
constexpr int kStateElems = 64 * 64 + 64;            // S then z of one head, d = 64; also one 64 x 64 quadrant + its z

// Workspace layout (B*H = BH heads, `elems` = d*d + d):
//   float  partial[BH][kMaxChunks][elems]
//   float  lookahead[BH][elems]       S then z per head: the updated state of a step that does not commit
//   u64    flags[BH][2][kMaxChunks]   epoch-tagged: [0] partial c stored, [1] slice c of the new state stored
//   u64    error, magic, pad, pad     error: kWsTimeoutMark once a bounded wait has timed out
//   u64    tickets[BH]                magic, tickets: device-side epochs (EpochSource), unused unless initialised
__host__ __device__ constexpr size_t ws_partial_bytes(int BH, int elems) {
    return (size_t)BH * kMaxChunks * elems * sizeof(float);
}
__host__ __device__ constexpr size_t ws_lookahead_bytes(int BH, int elems) {
    return (size_t)BH * elems * sizeof(float);
}
// S part of the look-ahead state ([BH][d*d]); the z part ([BH][d]) follows it.
__host__ __device__ __forceinline__ float *ws_lookahead(void *ws, int BH, int elems) {
    return reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + ws_partial_bytes(BH, elems));
}
__host__ __device__ __forceinline__ unsigned long long *ws_flag_base(void *ws, int BH, int elems) {
    return reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(ws) + ws_partial_bytes(BH, elems) +
                                                  ws_lookahead_bytes(BH, elems));
}
__host__ __device__ __forceinline__ unsigned long long *ws_flags(void *ws, int BH, int elems, int bh, int phase) {
    return ws_flag_base(ws, BH, elems) + ((size_t)bh * 2 + phase) * kMaxChunks;
}
__host__ __device__ constexpr size_t ws_error_offset(int BH, int elems) {
    return ws_partial_bytes(BH, elems) + ws_lookahead_bytes(BH, elems) + (size_t)BH * 2 * kMaxChunks * sizeof(unsigned long long);
}
__host__ __device__ __forceinline__ unsigned long long *ws_error(void *ws, int BH, int elems) {
    return reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(ws) + ws_error_offset(BH, elems));
}
__host__ __device__ __forceinline__ unsigned long long *ws_magic(void *ws, int BH, int elems) {
    return ws_error(ws, BH, elems) + 1;
}
__host__ __device__ __forceinline__ unsigned long long *ws_tickets(void *ws, int BH, int elems) {
    return ws_error(ws, BH, elems) + 4;
}
__host__ __device__ constexpr size_t ws_total_bytes(int BH, int elems) {
    return ws_partial_bytes(BH, elems) + ws_lookahead_bytes(BH, elems) +
           ((size_t)BH * 2 * kMaxChunks + 4 + (size_t)BH) * sizeof(unsigned long long);
}

// Where a launch gets the epoch that tags its flags.
//
// Normally the host draws a fresh one per call and passes it as a kernel
// argument.  A launch recorded in a HIP graph replays with the same arguments, so
// a workspace can be switched to device-side epochs instead: once its header holds
// kWsMagic (sv_linattn_workspace_init), every launch takes its epochs from ticket
// counters in the workspace, one per head (flags are per head, so only a head's
// workgroups have to agree).  Each workgroup of a head adds to the head's counter
// when it starts, workgroup 0 adding what is missing to kTicketQuantum in total;
// launches on a stream do not overlap, so all workgroups of the head's n-th
// launch draw tickets in [n * quantum, (n + 1) * quantum) and agree on n, however
// many workgroups each launch gave the head.  Nothing is ever reset.
// Device epochs are even, host epochs odd: they never collide.  A host epoch with its top bit set tells
// the kernel not to look for kWsMagic at all (kHostEpochsOnly: the workspace is memory whose header
// nobody can have initialised and whose contents, left by calls of other shapes, are arbitrary).
constexpr unsigned long long kWsMagic = 0x73764c696e417474ull;
// What the workspace's error word holds after a bounded wait has run out.  A fixed pattern, so that the
// word means something in a workspace whose contents were never initialised (any other value: no timeout).
constexpr unsigned long long kWsTimeoutMark = 0x54494d454f555421ull;
constexpr unsigned long long kTicketQuantum = 1ull << 20;     // far more than a head ever has workgroups
constexpr unsigned long long kHostEpochsOnly = 1ull << 63;

struct EpochSource {
    unsigned long long host, ticket, magic;    // ticket and magic are meaningful in thread 0 only

    // First thing in the kernel, in workgroup c of the C workgroups of head bh.  Nothing here looks at
    // what the two memory operations return, so the wave goes straight on to request its first tiles;
    // they have long returned when resolve() needs them.  The ticket is drawn whether or not the
    // workspace was initialised (the counters are reserved for this either way): deciding that first
    // would cost the wave a memory round trip before its first load.
    __device__ __forceinline__ void begin(void *ws, int BH, int elems, unsigned long long host_epoch, int bh, int c, int C)
    {
        host = host_epoch;
        ticket = 0;
        magic = 0;
        if (threadIdx.x == 0) {
            magic = __hip_atomic_load(ws_magic(ws, BH, elems), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned long long w = c == 0 ? kTicketQuantum - (unsigned long long)(C - 1) : 1ull;
            ticket = __hip_atomic_fetch_add(ws_tickets(ws, BH, elems) + bh, w, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // The launch's epoch for this head, in all threads.  Must be called by all threads
    // (one barrier); `lds_word` is 8 bytes of LDS that nothing else uses.
    __device__ __forceinline__ unsigned long long resolve(unsigned long long *lds_word) const
    {
        if (threadIdx.x == 0) {
            // What begin() fetched is looked at here and not before: without the two empty statements the
            // compiler moves this arithmetic up into begin()'s branch (same condition), and the wave then
            // waits for a device-scope atomic's round trip before it requests its first tile.
            unsigned long long m = magic, t = ticket;
            asm volatile("" : "+v"(m));
            asm volatile("" : "+v"(t));
            const bool device = m == kWsMagic && !(host & kHostEpochsOnly);
            *lds_word = device ? ((t / kTicketQuantum + 1) << 1) : host;
        }
        wg_barrier();
        return *lds_word;
    }
};

// Bytes of LDS that kernels with in-kernel waits append to their dynamic allocation for resolve().
constexpr int kEpochLdsBytes = 16;

// Registers of one lane: a 64x64 fp32 partial state as four 32x32 MFMA
// accumulators, S[32*rb + m][32*cb + n], and the key sums: as two more
// accumulators whose columns all hold sum_j phi(K[j][32*rb + m]) (plain
// kernels), or as 8 per-lane sums (RoPE kernels, where the keys that reach the
// MFMA are rotated but the key sum is not).
struct StateAcc {
    f32x16 s[2][2];   // [key feature block][value feature block]
    f32x16 zm[2];     // [key feature block]
    float z[8];       // features (lane%8)*8 + e of the tokens this lane loaded
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[rb][cb][i] = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) zm[rb][i] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = 0.f;
    }
};

// Coalesced load of a TILE x 64 bf16 tile: lane l takes bytes 16*(l%8) .. +16 of
// rows l/8 + 8i.  `off0` is the tile's byte offset (TileWalk::offset).
template <int TILE>
__device__ __forceinline__ void token_tile_load(rsrc_t r, uint32_t off0, uint32_t row_bytes, int lane,
                                                u32x4 (&reg)[TILE / 8])
{
    const uint32_t lane_off = (uint32_t)(lane >> 3) * row_bytes + (uint32_t)(lane & 7) * 16u;
#pragma unroll
    for (int i = 0; i < TILE / 8; ++i) reg[i] = load_stream16(r, off0 + lane_off + (uint32_t)i * 8u * row_bytes);
}

// MFMA operand from a token-major LDS tile: for the lane's MFMA row
// r = lane%32 and k-group g = lane/32, features f0 + r of tokens tok0 + 8g .. +8.
// Two transposing reads of four tokens each; within a block of 16 lanes, lane i
// supplies the address of token (i/4), features 4*(i%4) .. +4 of the block's 16.
template <int ROWB = kRowBytes>
__device__ __forceinline__ bf16x8 lds_tr_operand(const unsigned char *tile, int tok0, int f0, int lane)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    const int i = lane & 15, fb = (lane >> 4) & 1, g = lane >> 5;
    const unsigned char *p = tile + (tok0 + 8 * g + (i >> 2)) * ROWB + (f0 + 16 * fb + 4 * (i & 3)) * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * ROWB));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
}

// One wave's input stream: buffer resources over the head's K and V rows below
// the end of the token range, the wave's tile walk, the register staging of
// DEPTH tiles in flight, and the rotation source (ROPE: kRopeNone/Table/3D).
template <int TILE, int DEPTH, int ROPE>
struct StateStream {
    rsrc_t rK, rV;
    uint32_t row_bytes;
    int lane;
    TileWalk walk;
    u32x4 k[DEPTH][TILE / 8], v[DEPTH][TILE / 8];
    Rotator<ROPE, TILE / 8, DEPTH> rot;

    __device__ __forceinline__ StateStream(const uint16_t *Kh, const uint16_t *Vh, const RopeArg &rope,
                                           const unsigned char *lds_tab, int64_t stride_n, int t1, int lane_,
                                           const TileWalk &w)
        : rK(make_rsrc(Kh, (uint32_t)t1 * (uint32_t)stride_n * 2u)),
          rV(make_rsrc(Vh, (uint32_t)t1 * (uint32_t)stride_n * 2u)), row_bytes((uint32_t)stride_n * 2u), lane(lane_),
          walk(w), rot(rope, t1, 64, lane_ >> 3, 8, 4 * (lane_ & 7), 1, lds_tab) {}

    // Requests the wave's i-th tile into stage s.  Always the same number of memory
    // instructions: past the wave's share they read nothing and return zeros.
    __device__ __forceinline__ void request(int s, int i)
    {
        token_tile_load<TILE>(rK, walk.offset<TILE>(i, row_bytes), row_bytes, lane, k[s]);
        token_tile_load<TILE>(rV, walk.offset<TILE>(i, row_bytes), row_bytes, lane, v[s]);
        rot.request(s, i < walk.count, walk.token<TILE>(i));
    }
};

// Requests the first DEPTH tiles of a wave's share.
template <int TILE, int DEPTH, int ROPE>
__device__ __forceinline__ void state_prefetch(StateStream<TILE, DEPTH, ROPE> &st)
{
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
        st.request(s, s);
        __builtin_amdgcn_sched_barrier(0);   // requests go out in stage order, as they do in the loop
    }
}

// Accumulates the wave's share, whose first DEPTH tiles state_prefetch has
// requested.  Tiles are taken DEPTH at a time; in the last round the stages past
// the share hold zeros, as do tokens past t1, and add nothing to either sum.
// `tileK`/`tileV` are this wave's private LDS tiles.
template <int TILE, int DEPTH, int ROPE>
__device__ __forceinline__ void state_accumulate(StateStream<TILE, DEPTH, ROPE> &st, unsigned char *tileK,
                                                 unsigned char *tileV, int lane, StateAcc &acc)
{
    static_assert(TILE == 16 || TILE == 32, "tile is one or two MFMA k-steps");
    const int wr_off = (lane >> 3) * kRowBytes + (lane & 7) * 16;

    for (int i0 = 0; i0 < st.walk.count; i0 += DEPTH) {
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            // keep each stage's work together: a later stage's registers must not be touched (and
            // waited for) before this stage has been refilled
            __builtin_amdgcn_sched_barrier(0);
            // phi(K) on the packed pairs
            st.rot.template begin_tile<TILE>(st.walk, i0 + s);
            // the table lookups of the tile go out first; ReLU and key sums fill their latency
            f32x2 cs[TILE / 8][4];
#pragma unroll
            for (int i = 0; i < TILE / 8; ++i) st.rot.fetch(s, i, cs[i]);
#pragma unroll
            for (int i = 0; i < TILE / 8; ++i) {
                const u32x4 kk = relu_bf16x8(st.k[s][i]);
                if (ROPE) {
                    // the key sum is never rotated; the keys that meet V are (RoPE after ReLU)
                    acc.z[0] += bf16_lo(kk.x);  acc.z[1] += bf16_hi(kk.x);
                    acc.z[2] += bf16_lo(kk.y);  acc.z[3] += bf16_hi(kk.y);
                    acc.z[4] += bf16_lo(kk.z);  acc.z[5] += bf16_hi(kk.z);
                    acc.z[6] += bf16_lo(kk.w);  acc.z[7] += bf16_hi(kk.w);
                }
                st.k[s][i] = kk;
            }
#pragma unroll
            for (int i = 0; i < TILE / 8; ++i) st.k[s][i] = st.rot.rotate_with(st.k[s][i], cs[i]);
            wave_lds_fence();   // earlier reads of the tile buffer are done before it is overwritten
#pragma unroll
            for (int i = 0; i < TILE / 8; ++i) {
                *reinterpret_cast<u32x4 *>(tileK + wr_off + 8 * i * kRowBytes) = st.k[s][i];
                *reinterpret_cast<u32x4 *>(tileV + wr_off + 8 * i * kRowBytes) = st.v[s][i];
            }
            st.request(s, i0 + s + DEPTH);   // refill this stage: DEPTH tiles ahead
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_fence();
#pragma unroll
            for (int ks = 0; ks < TILE / 16; ++ks) {
                const bf16x8 a0 = lds_tr_operand(tileK, 16 * ks, 0, lane), a1 = lds_tr_operand(tileK, 16 * ks, 32, lane);
                const bf16x8 b0 = lds_tr_operand(tileV, 16 * ks, 0, lane), b1 = lds_tr_operand(tileV, 16 * ks, 32, lane);
                acc.s[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc.s[0][0], 0, 0, 0);
                acc.s[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc.s[0][1], 0, 0, 0);
                acc.s[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc.s[1][0], 0, 0, 0);
                acc.s[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc.s[1][1], 0, 0, 0);
                if (!ROPE) {
                    const uint32_t one2 = 0x3f803f80u;   // bf16 (1.0, 1.0)
                    const u32x4 ones4 = {one2, one2, one2, one2};
                    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones4);
                    acc.zm[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, ones, acc.zm[0], 0, 0, 0);
                    acc.zm[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, ones, acc.zm[1], 0, 0, 0);
                }
            }
        }
    }
}

// Lays one wave's accumulators out in [k][v] order (64 x 64 floats, then the 64
// key sums) in its LDS slot `dst`.  ZVALU: the key sums are the per-lane sums
// acc.z (RoPE kernels for d = 64), otherwise the accumulators acc.zm.
template <bool ZVALU>
__device__ __forceinline__ void state_acc_to_slot(StateAcc &acc, float *dst, int lane)
{
    // 32x32 accumulator layout: register i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32.
    // (one base address per lane and compile-time offsets from it: the 96 LDS writes then need no address arithmetic)
    const int n = lane & 31, g = lane >> 5;
    float *row0 = dst + (4 * g) * 64 + n, *z0 = dst + 64 * 64 + 4 * g;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int kc = 32 * rb + 8 * (i >> 2) + (i & 3);   // k = kc + 4 g
            row0[kc * 64] = acc.s[rb][0][i];
            row0[kc * 64 + 32] = acc.s[rb][1][i];
        }
    if (!ZVALU && n == 0) {                                  // every column of zm holds the key sums
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int i = 0; i < 16; ++i) z0[32 * rb + 8 * (i >> 2) + (i & 3)] = acc.zm[rb][i];
    }
    if (ZVALU) {
        // lanes with equal lane%8 hold the same 8 features (wavefront-level reduction)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = acc.z[e];
            x += __shfl_xor(x, 8);
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            acc.z[e] = x;
        }
        if (lane < 8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[64 * 64 + lane * 8 + e] = acc.z[e];
        }
    }
}

// d = 64: adds the WAVES waves' accumulators in a fixed tree order and stores the
// workgroup's partial state, S in [k][v] order followed by z, to `out`
// (kStateElems floats) with coherent stores spread over all threads: after one
// barrier each thread adds the waves' slots for its share of the elements,
// wave w absorbing wave w + h for h = WAVES/2, ..., 1.  Must be called by all
// threads; the staging tiles are dead afterwards.  LDS: WAVES * kStateElems floats.
template <int WAVES, bool ZVALU, bool LOCAL = false>
__device__ __forceinline__ void state_wg_reduce_store(StateAcc &acc, float *slots, int wave, int lane,
                                                      float *__restrict__ out)
{
    constexpr int THREADS = 64 * WAVES;
    wg_barrier();                                   // all waves are done with their staging tiles
    state_acc_to_slot<ZVALU>(acc, slots + wave * kStateElems, lane);
    wg_barrier();
    // a fixed number of rounds, all LDS reads of the workgroup's share issued before the first sum: this sits on
    // the chain of round trips by which a head agrees on its state
    constexpr int kUnits = kStateElems / 2, kRounds = (kUnits + THREADS - 1) / THREADS;
    f32x2 x[kRounds][WAVES];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        int v = (int)threadIdx.x + r * THREADS;
        v = v < kUnits ? v : kUnits - 1;                 // past the end: any valid unit, the sum is not stored
#pragma unroll
        for (int w = 0; w < WAVES; ++w) x[r][w] = *reinterpret_cast<const f32x2 *>(slots + w * kStateElems + 2 * v);
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
#pragma unroll
        for (int h = WAVES / 2; h >= 1; h /= 2)
#pragma unroll
            for (int w = 0; w < h; ++w) x[r][w] += x[r][w + h];
        const int v = (int)threadIdx.x + r * THREADS;
        if (v < kUnits) store_coherent<LOCAL>(out + 2 * v, x[r][0]);
    }
}

// d = 112, 128: wave w holds quadrant (key block w%2, value block w/2) of the
// workgroup's partial state; the four slots are stitched into the d x d matrix
// (row length d) followed by the d key sums (taken from the waves of value
// block 0) and stored to `out` (d*d + d floats) with coherent stores.
__device__ __forceinline__ void state_wg_quadrant_store(StateAcc &acc, float *slots, int wave, int lane, int d,
                                                        float *__restrict__ out)
{
    wg_barrier();                                   // all waves are done with their staging tiles
    state_acc_to_slot<false>(acc, slots + wave * kStateElems, lane);
    wg_barrier();
    const int s_units = d * d / 2, units = s_units + d / 2;
    for (int u = threadIdx.x; u < units; u += 4 * kWave) {
        const float *src;
        if (u < s_units) {
            const int k = (2 * u) / d, v = 2 * u - k * d;
            src = slots + ((k >> 6) + 2 * (v >> 6)) * kStateElems + (k & 63) * 64 + (v & 63);
        } else {
            const int k = 2 * (u - s_units);
            src = slots + (k >> 6) * kStateElems + 64 * 64 + (k & 63);
        }
        store_coherent(out + 2 * u, *reinterpret_cast<const f32x2 *>(src));
    }
}

// The carried values (S_in, z_in; zeros if S_in is null) of the units a thread folds first.  They do
// not depend on the other workgroups, so they are fetched before the wait for the partials, off
// the chain of round trips that follows it.
template <int THREADS, int UNITS>
__device__ __forceinline__ void state_slice_carry(const StateSlice &sl, const float *S_in, const float *z_in, int tid,
                                                  f32x2 (&x)[UNITS])
{
#pragma unroll
    for (int u = 0; u < UNITS; ++u) x[u] = f32x2{0.f, 0.f};
    if (S_in) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            int v = sl.lo + tid + u * THREADS;               // beyond the slice: any valid unit, the value is not used
            v = v < sl.units ? v : sl.units - 1;
            x[u] = *reinterpret_cast<const f32x2 *>(v < sl.s_units ? S_in + 2 * v : z_in + 2 * (v - sl.s_units));
        }
    }
}

//   S_out, z_out = (S_in, z_in or 0) + partial[0] + partial[1] + ... + partial[C-1], in that order,
// for the slice.  S_in may be null (no carried state) or equal to S_out (update in place); `carry`
// holds what state_slice_carry fetched.  Partials come in through coherent loads, GROUP chunks in
// flight per unit: the loads of a round trip of ~1 us are all issued before any is used.
// COHERENT_OUT: also store the result coherently (other workgroups of this kernel are going to
// read it).  Called by THREADS threads numbered tid = 0 .. THREADS - 1 (a workgroup, or one wave).
template <int THREADS, bool COHERENT_OUT, int UNITS = 3, int GROUP = 16, bool LOCAL = false>
__device__ __forceinline__ void state_finalize_slice(const float *__restrict__ partials, const StateSlice &sl, int C,
                                                     const float *S_in, const float *z_in, float *S_out,
                                                     float *z_out, int tid, const f32x2 (&carry)[UNITS])
{
    const int s_units = sl.s_units, elems = 2 * sl.units, hi = sl.hi;
    for (int v0 = sl.lo + tid; v0 < hi; v0 += THREADS * UNITS) {
        f32x2 x[UNITS];
#pragma unroll
        for (int u = 0; u < UNITS; ++u) x[u] = carry[u];
        if (v0 != sl.lo + tid) {                                 // slices longer than one round: fetched here
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                const int v = v0 + u * THREADS;
                x[u] = f32x2{0.f, 0.f};
                if (S_in && v < hi) x[u] = *reinterpret_cast<const f32x2 *>(v < s_units ? S_in + 2 * v : z_in + 2 * (v - s_units));
            }
        }
        // Straight-line loads: a wave-uniform base per partial plus one 32-bit offset per unit, no branch (a group
        // that reaches past C re-reads the last partial and leaves it out of the sum).  This runs on the chain of
        // round trips by which a head agrees on its state, where every instruction counts.
        uint32_t off[UNITS];
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            int v = v0 + u * THREADS;                            // beyond the slice: any valid unit, the sum is not stored
            v = v < sl.units ? v : sl.units - 1;
            off[u] = 2u * (uint32_t)v;
        }
        for (int c0 = 0; c0 < C; c0 += GROUP) {
            f32x2 p[UNITS][GROUP];
#pragma unroll
            for (int cc = 0; cc < GROUP; ++cc) {
                const float *part = partials + (size_t)(c0 + cc < C ? c0 + cc : C - 1) * elems;
#pragma unroll
                for (int u = 0; u < UNITS; ++u) p[u][cc] = load_coherent(part + off[u]);
            }
#pragma unroll
            for (int u = 0; u < UNITS; ++u)
#pragma unroll
                for (int cc = 0; cc < GROUP; ++cc)
                    if (c0 + cc < C) x[u] += p[u][cc];
        }
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int v = v0 + u * THREADS;
            if (v < hi) {
                float *dst = v < s_units ? S_out + 2 * v : z_out + 2 * (v - s_units);
                if (COHERENT_OUT) store_coherent<LOCAL>(dst, x[u]);
                else *reinterpret_cast<f32x2 *>(dst) = x[u];
            }
        }
    }
}

// The calling workgroup has just issued coherent stores that belong to phase
// `phase` (0: partial c, 1: slice c of the new state) of head `bh`: publish them.
// All threads must call.
__device__ __forceinline__ void state_publish(void *ws, int BH, int elems, int bh, int c, int phase,
                                              unsigned long long epoch)
{
    coherent_stores_done();                             // this wave's stores are performed
    wg_barrier();
    if (threadIdx.x == 0) flag_publish(ws_flags(ws, BH, elems, bh, phase) + c, epoch);
}

// Waits until all C workgroups of head `bh` have published `phase`.  Returns
// false (and records it in the workspace) if the bounded wait ran out: the caller
// must then store nothing that depends on the other workgroups.  The result is
// uniform over the calling wave.
__device__ __forceinline__ bool state_wait(void *ws, int BH, int elems, int bh, int C, int phase,
                                           unsigned long long epoch, uint32_t spin_limit, int lane)
{
    const bool ok = flags_wait_all(ws_flags(ws, BH, elems, bh, phase), C, epoch, spin_limit, lane);
    if (!ok && lane == 0)
        __hip_atomic_store(ws_error(ws, BH, elems), kWsTimeoutMark, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return ok;
}

__device__ __forceinline__ bool state_publish_and_wait(void *ws, int BH, int elems, int bh, int c, int C, int phase,
                                                       unsigned long long epoch, uint32_t spin_limit, int lane)
{
    state_publish(ws, BH, elems, bh, c, phase, epoch);
    return state_wait(ws, BH, elems, bh, C, phase, epoch, spin_limit, lane);
}

// Dynamic LDS of state_mfma: staging tiles or reduction slots.
template <int TILE, int WAVES>
__host__ __device__ constexpr int state_lds_bytes() {
    constexpr int stage = WAVES * 2 * TILE * kRowBytes, red = WAVES * kStateElems * 4;
    return (stage > red ? stage : red) + kEpochLdsBytes;
}

// grid = (C, B*H), block = 64*WAVES.  Wave w of workgroup c owns tiles
// WAVES*c + w + WAVES*C*i (i = 0, 1, ...) of the T = ceil((t1-t0)/TILE) tiles.
// FINALIZE: the C workgroups of a head wait for each other's partials and each
// folds one slice of them: S_out, z_out = (S_in, z_in, or 0 if S_in is null) +
// partials; this needs the whole grid to be resident.
// Otherwise only the partials are written and state_reduce finishes the job.
// ROPE (kRopeNone/Table/3D): keys are rotated before they meet V; with kRope3D the dynamic LDS
// carries kRope3dLdsBytes more for the tables.
template <int TILE, int WAVES, int DEPTH, bool FINALIZE, int ROPE>
__global__ __launch_bounds__(64 * WAVES, 1) void state_mfma_d64(
    const uint16_t *__restrict__ K, const uint16_t *__restrict__ V, RopeArg rope, TokStrides st,
    int H, int /* d: always 64; keeps the argument list of the d = 112/128 kernel */, int t0, int t1,
    int C, const float *S_in, const float *z_in, float *S_out, float *z_out, void *__restrict__ ws,
    unsigned long long epoch, uint32_t spin_limit)
{
    constexpr int THREADS = 64 * WAVES;
    constexpr int kTileBytes = TILE * kRowBytes;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x, bh = blockIdx.y, BH = gridDim.y;
    const int b = bh / H, h = bh % H;
    const uint16_t *Kh = K + b * st.b + h * st.h;
    const uint16_t *Vh = V + b * st.b + h * st.h;
    const int n_tiles = (t1 - t0 + TILE - 1) / TILE;
    EpochSource es;
    if (FINALIZE) es.begin(ws, BH, kStateElems, epoch, bh, c, C);

    StateAcc acc;
    acc.clear();
    const unsigned char *lds_tab = lds + state_lds_bytes<TILE, WAVES>();
    StateStream<TILE, DEPTH, ROPE> stream(Kh, Vh, rope, lds_tab, st.n, t1, lane,
                                          TileWalk(t0, WAVES * c + wave, WAVES * C, n_tiles, bh));
    unsigned char *tileK = lds + wave * 2 * kTileBytes;
    Rope3dFill tabs;
    if (ROPE == kRope3D) rope3d_lds_fill_begin(rope.r3, tabs);   // the first loads of the kernel
    state_prefetch(stream);
    if (ROPE == kRope3D) {
        rope3d_lds_fill_end(lds + state_lds_bytes<TILE, WAVES>(), rope.r3, tabs);
        wg_barrier();
    }
    state_accumulate(stream, tileK, tileK + kTileBytes, lane, acc);

    float *partials = static_cast<float *>(ws) + (size_t)bh * kMaxChunks * kStateElems;
    state_wg_reduce_store<WAVES, ROPE != kRopeNone>(acc, reinterpret_cast<float *>(lds), wave, lane,
                                                    partials + (size_t)c * kStateElems);
    if (FINALIZE) {
        epoch = es.resolve(reinterpret_cast<unsigned long long *>(lds + state_lds_bytes<TILE, WAVES>() - kEpochLdsBytes));
        const float *Sc = S_in ? S_in + (size_t)bh * 64 * 64 : nullptr, *zc = z_in + (size_t)bh * 64;
        const StateSlice sl(c, C, 64);
        f32x2 carry[3];
        state_slice_carry<THREADS>(sl, Sc, zc, tid, carry);
        if (!state_publish_and_wait(ws, BH, kStateElems, bh, c, C, 0, epoch, spin_limit, lane))
            return;                                     // timed out: this wave leaves its part of S, z as it was
        state_finalize_slice<THREADS, false>(partials, sl, C, Sc, zc, S_out + (size_t)bh * 64 * 64,
                                             z_out + (size_t)bh * 64, tid, carry);
    }
}

}  // namespace sv
