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
// order, publishes again, and waits for the other slices, with its first Q
// tiles already in flight.  Every wait polls a bounded number of times, so
// every wave always reaches the end of the kernel.  Then all workgroups apply
// the new state to their share of Q_b.  The dependency
// "all of the block's keys before any of its outputs" is per head, not grid
// wide, so heads drift past each other and reads overlap writes.
#pragma once

#include "apply_mfma.hpp"
#include "state_mfma.hpp"

namespace sv {

template <int DP, int TILE, int WAVES, bool ROPE>
__host__ __device__ constexpr int block_step_lds_bytes() {
    return state_lds_bytes<TILE, WAVES>() > apply_lds_bytes<DP, WAVES, ROPE>() ? state_lds_bytes<TILE, WAVES>()
                                                                               : apply_lds_bytes<DP, WAVES, ROPE>();
}

// grid = (C, B*H) with C*B*H <= resident workgroup capacity, block = 64*WAVES.
// DP = 64 serves d = 64, DP = 128 serves d = 112 and 128 (waves split features as
// in state_mfma and apply_mfma).
// ROPE: keys and queries are rotated after the ReLU in the numerator path (table row = token of the block).
template <int DP, int TILE, int WAVES, int DEPTH_S, bool HILO, int DEPTH_A, bool ROPE>
__global__ __launch_bounds__(64 * WAVES, 1) void block_step_mfma(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    uint16_t *__restrict__ O, const float *__restrict__ rope, TokStrides st, int H, int d_arg, int N, int C,
    const float *S_in, const float *z_in, float *S_out, float *z_out, float eps, void *__restrict__ ws,
    unsigned long long epoch, uint32_t spin_limit)
{
    static_assert(TILE == kApplyTile, "both phases walk tiles of the same size");
    constexpr int THREADS = 64 * WAVES;
    constexpr int kTileBytes = TILE * kRowBytes;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = blockIdx.x, bh = blockIdx.y, BH = gridDim.y;
    const int b = bh / H, h = bh % H;
    const int d = DP == 64 ? 64 : d_arg, elems = d * d + d;
    const int64_t head_off = b * st.b + h * st.h;
    const int n_tiles = (N + TILE - 1) / TILE;
    // the carried state is read from S_in, z_in and the updated one written to S_out, z_out: the same
    // arrays when the step commits, a scratch copy when it only looks ahead
    const float *Sc = S_in + (size_t)bh * d * d, *zc = z_in + (size_t)bh * d;
    float *Sh = S_out + (size_t)bh * d * d, *zh = z_out + (size_t)bh * d;

    // ---- this wave's first two tiles of Q_b are requested right away: they arrive during the state
    //      phase and make no later load wait behind them ---------------------------------------------
    const ApplySplit<DP, WAVES> asplit(c, C, wave);
    constexpr int kEarly = DEPTH_A < 2 ? DEPTH_A : 2;
    ApplyStream<DP, DEPTH_A, ROPE> qstream(Q + head_off, O + head_off, rope, st.n, N, d, asplit.vb, lane,
                                           TileWalk(0, asplit.first, asplit.step, n_tiles, bh));
    apply_prefetch<0, kEarly>(qstream);

    // ---- fold this workgroup's share of K_b, V_b ------------------------------------------------
    {
        const StateSplit<DP, WAVES> ssplit(c, C, wave);
        StateAcc acc;
        acc.clear();
        StateStream<TILE, DEPTH_S, ROPE, DP == 64> kvstream(K + head_off, V + head_off, rope, st.n, N, d, ssplit.kb, ssplit.vb,
                                                  lane, TileWalk(0, ssplit.first, ssplit.step, n_tiles, bh));
        unsigned char *tileK = lds + wave * 2 * kTileBytes;
        state_prefetch(kvstream);
        state_accumulate(kvstream, tileK, tileK + kTileBytes, lane, ssplit.vb == 0, acc);
        // the rest of this wave's Q prefetch streams in while the head's state is being agreed on
        apply_prefetch<kEarly, DEPTH_A>(qstream);
        float *partials = static_cast<float *>(ws) + (size_t)bh * kMaxChunks * elems;
        if (DP == 64)
            state_wg_reduce_store<WAVES, ROPE>(acc, reinterpret_cast<float *>(lds), wave, lane,
                                         partials + (size_t)c * elems);
        else
            state_wg_quadrant_store<ROPE>(acc, reinterpret_cast<float *>(lds), wave, lane, d, partials + (size_t)c * elems);
    }

    // ---- once all partials of the head are there, fold this workgroup's slice into S, z in place,
    //      then wait for the other slices -------------------------------------------------------
    {
        const float *partials = static_cast<const float *>(ws) + (size_t)bh * kMaxChunks * elems;
        state_publish_and_wait(ws, BH, elems, bh, c, C, 0, epoch, spin_limit, lane);
        state_finalize_slice<THREADS, true>(partials, c, C, d, Sc, zc, Sh, zh);
        state_publish_and_wait(ws, BH, elems, bh, c, C, 1, epoch, spin_limit, lane);
    }

    // ---- apply the updated state to this workgroup's share of Q_b ----------------------------------
    ApplyOperands<DP, HILO> A;
    A.template load<true>(Sh, zh, d, asplit.vb, lane);
    apply_tiles<DP, HILO>(qstream, lds + wave * apply_wave_lds_bytes<DP, ROPE>(), lane, A, eps);
}

}  // namespace sv
