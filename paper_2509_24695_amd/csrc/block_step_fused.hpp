// One-launch block step for d = 64 bf16 on gfx950 (Sec. 3.3.1; cache update and
// use of Alg. 1):
//
//   S += phi(K_b)^T V_b,  z += sum phi(K_b),  O_b = phi(Q_b) S / (phi(Q_b) z + eps)
//
// with O_b computed from the UPDATED state.  The grid is sized so that every
// workgroup is resident at once (one per compute unit).  Each workgroup first
// reduces its round-robin share of the block's keys and values to a partial
// state and publishes it with an epoch-tagged flag; when all partials of its
// head are there it folds one slice of them into the carried S, z in chunk
// order, publishes again, and waits for the other slices (one wave does this,
// the others have their first Q tiles in flight meanwhile).  Every wait polls a
// bounded number of times, so every wave always reaches the end of the kernel.
// Then all workgroups apply the new state to their share of Q_b.  The
// dependency "all of the block's keys before any of its outputs" is per head,
// not grid wide, so heads drift past each other and reads overlap writes.
#pragma once

#include "apply_mfma.hpp"
#include "state_mfma.hpp"

namespace sv {

template <int TILE, int WAVES, int ROPE>
__host__ __device__ constexpr int block_step_lds_bytes() {
    constexpr int s = state_lds_bytes<TILE, WAVES>();
    constexpr int a = apply_lds_bytes<WAVES, ROPE>() + kEpochLdsBytes;
    return s > a ? s : a;   // both include the epoch word, which sits at the very end
}

// grid = (C, B*H) with C*B*H <= resident workgroup capacity, block = 64*WAVES.  Waves work alone,
// as in state_mfma_d64 and apply_mfma_d64.  (d = 112 and 128 take the step as two launches: there
// the state and the apply kernel want different workgroup shapes, and one launch measured 2-8 us
// slower at every block size.)
// ROPE: keys and queries are rotated after the ReLU in the numerator path (table row = token of the block).
// LOCAL: grid = (C * B*H) with B*H a multiple of n_dies; all workgroups of a head run on one die and
// exchange their partial states and the new state through that die's L2 (see store_coherent).
template <int TILE, int WAVES, int DEPTH_S, bool HILO, int DEPTH_A, int ROPE, bool LOCAL = false, bool DEN_VALU = false>
__global__ __launch_bounds__(64 * WAVES, 1) void block_step_mfma(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    uint16_t *__restrict__ O, RopeArg rope, TokStrides st, int H, int N, int C,
    const float *S_in, const float *z_in, float *S_out, float *z_out, float eps, void *__restrict__ ws,
    unsigned long long epoch, uint32_t spin_limit, int BH_local, int n_dies)
{
    static_assert(TILE == kApplyTile, "both phases walk tiles of the same size");
    // Every argument is fetched with the first batch of scalar loads.  Left alone the compiler fetches
    // some of them where they are first used - K and V right before the first tile request, the state pointers in
    // the middle of the agreement chain - and each such fetch is a round trip nobody can hide.
    asm volatile("" ::"s"(Q), "s"(K), "s"(V), "s"(O), "s"(S_in), "s"(z_in), "s"(S_out), "s"(z_out), "s"(ws), "s"(epoch),
                 "s"(eps), "s"(spin_limit));
    constexpr int kTileBytes = TILE * kRowBytes;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int c = blockIdx.x, bh = blockIdx.y, BH = gridDim.y;
    if (LOCAL) {
        // consecutive workgroup ids go round the dies: die x gets ids x, x + n_dies, ..., and with them
        // heads x, x + n_dies, ..., C workgroups each
        const int die = (int)blockIdx.x % n_dies, slot = (int)blockIdx.x / n_dies;
        BH = BH_local;
        bh = die + n_dies * (slot / C);
        c = slot % C;
    }
    const uint32_t my_die = LOCAL ? die_id() : 0u;
    const int b = bh / H, h = bh % H;
    constexpr int d = 64, elems = d * d + d;
    const int64_t head_off = b * st.b + h * st.h;
    const int n_tiles = (N + TILE - 1) / TILE;
    // the carried state is read from S_in, z_in and the updated one written to S_out, z_out: the same
    // arrays when the step commits, a scratch copy when it only looks ahead
    const float *Sc = S_in + (size_t)bh * d * d, *zc = z_in + (size_t)bh * d;
    float *Sh = S_out + (size_t)bh * d * d, *zh = z_out + (size_t)bh * d;
    float *partials = static_cast<float *>(ws) + (size_t)bh * kMaxChunks * elems;
    EpochSource es;
    es.begin(ws, BH, elems, epoch, bh, c, C);
    // kRope3D: the tables sit behind everything else in LDS and live through both phases
    const unsigned char *lds_tab = lds + block_step_lds_bytes<TILE, WAVES, ROPE>();

    // ---- this wave's first two tiles of Q_b are requested right away: they arrive during the
    //      state phase and make no later load wait behind them --------------------------------
    constexpr int kEarly = DEPTH_A < 2 ? DEPTH_A : 2;
    // Shares are dealt to the workgroups starting at a different one in each head: when the tiles do not
    // divide evenly the longer shares fall on low share numbers, and workgroup c of every head runs on
    // the same die (consecutive workgroup ids go round the dies).
    const int share = block_step_share(c, bh, C);
    const int phase_key = LOCAL ? die_local_phase_key(bh, n_dies, BH) : bh;   // heads start their walks at staggered phases
    const TileWalk walk(0, WAVES * share + wave, WAVES * C, n_tiles, phase_key);
    ApplyStream<DEPTH_A, ROPE> qstream(Q + head_off, O + head_off, rope, lds_tab, st.n, N, lane, walk);
    Rope3dFill tabs;
    if (ROPE == kRope3D) rope3d_lds_fill_begin(rope.r3, tabs);   // the first loads of the kernel
    apply_prefetch<0, kEarly>(qstream);

    // ---- fold this workgroup's share of K_b, V_b ----------------------------------------------
    unsigned char *epoch_lds = lds + block_step_lds_bytes<TILE, WAVES, ROPE>() - kEpochLdsBytes;
    {
        StateAcc acc;
        acc.clear();
        StateStream<TILE, DEPTH_S, ROPE> kvstream(K + head_off, V + head_off, rope, lds_tab, st.n, N, lane, walk);
        unsigned char *tileK = lds + wave * 2 * kTileBytes;
        state_prefetch(kvstream);
        if (ROPE == kRope3D) {
            rope3d_lds_fill_end(lds + block_step_lds_bytes<TILE, WAVES, ROPE>(), rope.r3, tabs);
            wg_barrier();
        }
        state_accumulate(kvstream, tileK, tileK + kTileBytes, lane, acc);
        state_wg_reduce_store<WAVES, ROPE != kRopeNone, LOCAL>(acc, reinterpret_cast<float *>(lds), wave, lane,
                                           partials + (size_t)share * elems);   // slot = share: the fold adds the shares in tile order
    }
    // ---- the head agrees on its new state ------------------------------------------------------
    // Wave 0 alone waits for the head's partials, folds this workgroup's slice into S, z, publishes
    // it and waits for the other slices: a chain of memory round trips.  The other waves request the
    // rest of their Q prefetch meanwhile (wave 0 after the chain): memory operations of a wave
    // complete in order, so the chain's wave keeps its own queue empty, and one wave per workgroup
    // polling is a quarter of the flag traffic.  The carried values of the slice are fetched before
    // the wait; they do not depend on the other workgroups.
    epoch = es.resolve(reinterpret_cast<unsigned long long *>(epoch_lds));
    int *agreed = reinterpret_cast<int *>(epoch_lds + 8);          // did both waits end in time?
    const StateSlice sl(c, C, d);
    f32x2 carry[5] = {};
    if (wave == 0) state_slice_carry<kWave>(sl, Sc, zc, lane, carry);
    if (LOCAL) {
        coherent_stores_done();
        wg_barrier();
        if (threadIdx.x == 0) flag_publish<true>(ws_flags(ws, BH, elems, bh, 0) + c, flag_with_die(epoch, my_die));
    } else {
        state_publish(ws, BH, elems, bh, c, 0, epoch);
    }
    if (wave != 0) {
        apply_prefetch<kEarly, DEPTH_A>(qstream);
    } else {
        bool same_die = true;
        bool ok = LOCAL ? flags_wait_all_local(ws_flags(ws, BH, elems, bh, 0), C, epoch, spin_limit, lane, my_die, &same_die)
                        : state_wait(ws, BH, elems, bh, C, 0, epoch, spin_limit, lane);
        ok = ok && same_die;
        if (ok) {
            state_finalize_slice<kWave, true, 5, 8, LOCAL>(partials, sl, C, Sc, zc, Sh, zh, lane, carry);
            coherent_stores_done();
            if (lane == 0) {
                if (LOCAL) flag_publish<true>(ws_flags(ws, BH, elems, bh, 1) + c, flag_with_die(epoch, my_die));
                else flag_publish(ws_flags(ws, BH, elems, bh, 1) + c, epoch);
            }
            ok = LOCAL ? flags_wait_all_local(ws_flags(ws, BH, elems, bh, 1), C, epoch, spin_limit, lane, my_die, &same_die)
                       : state_wait(ws, BH, elems, bh, C, 1, epoch, spin_limit, lane);
        }
        if (LOCAL && !ok && lane == 0)
            __hip_atomic_store(ws_error(ws, BH, elems), kWsTimeoutMark, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane == 0) *agreed = ok;
    }
    wg_barrier();
    // A wait that ran out (recorded in the workspace): nothing more is stored, neither this workgroup's
    // slice of S, z (if the first wait failed) nor any row of O_b.
    if (!*agreed) return;

    // ---- apply the updated state to this workgroup's share of Q_b --------------------------------
    ApplyOperands<64, HILO> A;
    static_assert(WAVES == 4 && block_step_lds_bytes<TILE, WAVES, ROPE>() >= ApplyOperands<64, HILO>::kSharedBytes + kEpochLdsBytes,
                  "LDS can stage S for load_shared");
    A.template load_shared<true>(Sh, zh, wave, lane, lds);   // through LDS that the state phase has left and the apply phase not yet taken
    float zf[4][8];
    if (DEN_VALU) load_key_sums<true>(zh, lane, zf);
    if (wave == 0) apply_prefetch<kEarly, DEPTH_A>(qstream);
    apply_tiles<HILO, DEPTH_A, ROPE, false, DEN_VALU>(qstream, lds + wave * apply_wave_lds_bytes<ROPE>(), lane, A, eps, nullptr, zf);
}

}  // namespace sv
