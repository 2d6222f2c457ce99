// Which token tiles a wave visits, and in which order.  Plain C++ (no device code): shared by the
// kernels and a host-side coverage test.
#pragma once

#include <stdint.h>

#ifndef SV_HOST_DEVICE
#if defined(__HIPCC__)
#define SV_HOST_DEVICE __host__ __device__
#else
#define SV_HOST_DEVICE
#endif
#endif

namespace sv {

constexpr uint32_t kOutOfRange = 0x80000000u;   // a byte offset no buffer resource built by the kernels covers

// Byte offset of the first row of the tile that starts at token `tok0`, or kOutOfRange.
SV_HOST_DEVICE inline uint32_t tile_offset(bool valid, int tok0, uint32_t row_bytes) {
    return valid ? (uint32_t)tok0 * row_bytes : kOutOfRange;
}

// A wave's share of the tiles that cover the token range [t0, t1): tiles
// first + j*step for j = 0 .. count-1 (all values wave-uniform), visited in the
// cyclic order j = rot, rot+1, .., count-1, 0, .., rot-1.  Heads start at
// different phases of their shares, head bh at (bh mod 16)/16: when all heads
// march through memory in lockstep, some sequence lengths put their streams on
// the same DRAM resources at the same time (N = 75 600, 64 heads: apply 290 us
// in lockstep, 246 us staggered; no length measured got slower).
struct TileWalk {
    int t0, first, step, count, rot;
    SV_HOST_DEVICE inline TileWalk(int t0_, int first_, int step_, int n_tiles, int bh)
        : t0(t0_), first(first_), step(step_),
          count(first_ < n_tiles ? (n_tiles - first_ + step_ - 1) / step_ : 0), rot(((bh & 15) * count) >> 4) {}
    // first token of the i-th tile the wave visits (TILE tokens per tile), i < count
    template <int TILE> SV_HOST_DEVICE inline int token(int i) const {
        int j = i + rot;
        j = j >= count ? j - count : j;
        return t0 + (first + j * step) * TILE;
    }
    // its byte offset for rows of row_bytes bytes, kOutOfRange past the share
    template <int TILE> SV_HOST_DEVICE inline uint32_t offset(int i, uint32_t row_bytes) const {
        return tile_offset(i < count, token<TILE>(i), row_bytes);
    }
};

// Slice c of a head's state when C workgroups fold it together: 8-byte units [lo, hi) of the
// d*d/2 + d/2 units that S (d x d floats) and z (d floats) make, per = ceil(units / C) each; late
// slices may be short or empty.
struct StateSlice {
    int s_units, units, lo, hi;
    SV_HOST_DEVICE inline StateSlice(int c, int C, int d) : s_units(d * d / 2), units(d * d / 2 + d / 2), lo(0), hi(0)
    {
        const int per = (units + C - 1) / C;
        lo = c * per < units ? c * per : units;
        hi = lo + per < units ? lo + per : units;
    }
};

// The share of the token tiles that workgroup c of head bh takes in the one-launch block step:
// dealt from a different start in each head (see block_step_mfma).
SV_HOST_DEVICE inline int block_step_share(int c, int bh, int C) { return (c + bh) % C; }

// Phase key (the `bh` argument of TileWalk) of head bh in the die-local forms of the kernels, where die x
// holds heads x, x + n_dies, ...: keyed by the head index itself, heads of one die would share phases (two
// distinct ones for four heads), so the sixteen phases are dealt die by die, the heads of a die as far apart
// as their number allows.
SV_HOST_DEVICE inline int die_local_phase_key(int bh, int n_dies, int BH)
{
    const int per_die = BH / n_dies > 0 ? BH / n_dies : 1;
    const int stride = per_die < 16 ? 16 / per_die : 1;
    return ((bh / n_dies) * stride + (bh % n_dies) % stride) & 15;
}

}  // namespace sv
