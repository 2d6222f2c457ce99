// RoPE after ReLU (numerator of the Sec. 3.2 equation): where the (cos, sin)
// entries of a token tile come from.
//
//   kRopeNone   no rotation (the plain entry points);
//   kRopeTable  a caller-made table, fp32 [N][d/2][2], read with the tile: its rows
//               are as long as the token's K and V rows together, and although all
//               heads share them (they come from HBM once) every wave has to pull
//               its rows through the caches;
//   kRope3D     3-D rotary embedding in factored form: pair p is turned by the frame,
//               the row or the column position of the token, so three small tables
//               (frames x n_t, rows x n_h, cols x n_w entries) say everything.  They
//               are copied into LDS once per workgroup and looked up per pair:
//               the token loops then issue no memory instruction for the rotation
//               and the kernel's traffic stays at the four token streams.
//
// All kernels apply the rotation in the coalesced register layout of a freshly
// loaded tile, where a 32-bit word is exactly one feature pair (2p, 2p+1) and a
// lane's 16-byte chunk holds four consecutive pairs of one token.
#pragma once

#include "common.hpp"

namespace sv {

constexpr int kRopeNone = 0, kRopeTable = 1, kRope3D = 2;

// Factored 3-D rotary tables (device pointers): [frames][n_t][2], [rows][n_h][2],
// [cols][n_w][2] fp32 (cos, sin).  Token t sits at frame t / (rows*cols), row
// (t / cols) % rows, column t % cols; pairs [0, n_t) follow the frame, pairs
// [n_t, n_t + n_h) the row, the rest the column.
struct Rope3D {
    const float *cs_t, *cs_h, *cs_w;
    int frames, rows, cols, n_t, n_h, n_w;
};

// Kernel argument of every mode.
struct RopeArg {
    const float *table;   // kRopeTable
    Rope3D r3;            // kRope3D
};

constexpr int kRope3dLdsBytes = 32768;   // LDS reserved for the three tables (the host checks that they fit)

__host__ __device__ constexpr int rope3d_entries(int frames, int rows, int cols, int n_t, int n_h, int n_w) {
    return frames * n_t + rows * n_h + cols * n_w;
}

// Copies the three tables to LDS, frame table first, in two parts so that the table reads can be
// the first memory operations of a kernel: _begin issues the loads of the first kRope3dFillBatch
// entries per thread (all of them, for tables of up to 16 KB and 256 threads) without waiting,
// the caller then requests its first token tiles, and _end stores to LDS (and copies whatever
// is left).  Memory operations return in order, so the tables are there before the tiles and the
// copy costs no round trip of its own.  All threads of the workgroup call both; the caller places
// a workgroup barrier between _end and the first lookup.
constexpr int kRope3dFillBatch = 8;
struct Rope3dFill {
    f32x2 v[kRope3dFillBatch];
};
// Entry e (clamped into range) of the three tables laid end to end.
__device__ __forceinline__ f32x2 rope3d_entry_flat(const Rope3D &R, int nt, int nh, int total, int e)
{
    e = e < total ? e : total - 1;
    const f32x2 *src = e < nt ? reinterpret_cast<const f32x2 *>(R.cs_t) + e
                              : (e < nt + nh ? reinterpret_cast<const f32x2 *>(R.cs_h) + (e - nt)
                                             : reinterpret_cast<const f32x2 *>(R.cs_w) + (e - nt - nh));
    return *src;
}
__device__ __forceinline__ void rope3d_lds_fill_begin(const Rope3D &R, Rope3dFill &f)
{
    const int nt = R.frames * R.n_t, nh = R.rows * R.n_h, total = nt + nh + R.cols * R.n_w;
#pragma unroll
    for (int j = 0; j < kRope3dFillBatch; ++j)
        f.v[j] = rope3d_entry_flat(R, nt, nh, total, (int)threadIdx.x + j * (int)blockDim.x);
}
__device__ __forceinline__ void rope3d_lds_fill_end(unsigned char *lds_tab, const Rope3D &R, const Rope3dFill &f)
{
    f32x2 *dst = reinterpret_cast<f32x2 *>(lds_tab);
    const int nt = R.frames * R.n_t, nh = R.rows * R.n_h, total = nt + nh + R.cols * R.n_w;
#pragma unroll
    for (int j = 0; j < kRope3dFillBatch; ++j) {
        const int e = (int)threadIdx.x + j * (int)blockDim.x;
        if (e < total) dst[e] = f.v[j];
    }
    for (int e = (int)threadIdx.x + kRope3dFillBatch * (int)blockDim.x; e < total; e += (int)blockDim.x)
        dst[e] = rope3d_entry_flat(R, nt, nh, total, e);
}

// One (cos, sin) entry straight from global memory (plain-FMA kernels).
__device__ __forceinline__ f32x2 rope3d_entry_global(const Rope3D &R, int tok, int p)
{
    const int rc = R.rows * R.cols;
    const int f = tok / rc, rem = tok - f * rc, r = rem / R.cols, c = rem - r * R.cols;
    if (p < R.n_t) return reinterpret_cast<const f32x2 *>(R.cs_t)[f * R.n_t + p];
    if (p < R.n_t + R.n_h) return reinterpret_cast<const f32x2 *>(R.cs_h)[r * R.n_h + (p - R.n_t)];
    return reinterpret_cast<const f32x2 *>(R.cs_w)[c * R.n_w + (p - R.n_t - R.n_h)];
}

// Rotation source of one wave's token stream.
//   STEPS  16-byte chunks a lane holds per tile (rows row0 + j * rows_per_step, j < STEPS)
//   DEPTH  tiles in flight (kRopeTable keeps their table rows in registers)
template <int MODE, int STEPS, int DEPTH>
struct Rotator;

template <int STEPS, int DEPTH>
struct Rotator<kRopeNone, STEPS, DEPTH> {
    __device__ __forceinline__ Rotator(const RopeArg &, int, int, int, int, int, int, const unsigned char *) {}
    __device__ __forceinline__ void request(int, bool, int) {}
    template <int TILE> __device__ __forceinline__ void begin_tile(const TileWalk &, int) {}
    __device__ __forceinline__ u32x4 rotate(int, int, u32x4 w) const { return w; }
    __device__ __forceinline__ void fetch(int, int, f32x2 (&)[4]) const {}
    __device__ __forceinline__ u32x4 rotate_with(u32x4 w, const f32x2 (&)[4]) const { return w; }
};

template <int STEPS, int DEPTH>
struct Rotator<kRopeTable, STEPS, DEPTH> {
    rsrc_t rT;
    uint32_t table_row_bytes, lane_off, step_bytes;
    f32x4 cs[DEPTH][STEPS][2];

    // t1: end of the token range; d: head dimension; row0, rows_per_step: the lane's rows of a
    // tile; pair0: first of the lane's four consecutive pairs; lane_valid: the pairs exist.
    __device__ __forceinline__ Rotator(const RopeArg &a, int t1, int d, int row0, int rows_per_step, int pair0,
                                       int /*lane_valid*/, const unsigned char *)
        : rT(make_rsrc(a.table, (uint32_t)t1 * (uint32_t)d * 4u)), table_row_bytes((uint32_t)d * 4u),
          lane_off((uint32_t)row0 * (uint32_t)d * 4u + (uint32_t)pair0 * 8u),
          step_bytes((uint32_t)rows_per_step * (uint32_t)d * 4u) {}

    // Requests the table rows of the tile that starts at token tok0 into stage s (nothing
    // is read if !valid: out-of-range offsets return zeros).
    __device__ __forceinline__ void request(int s, bool valid, int tok0)
    {
        const uint32_t off0 = tile_offset(valid, tok0, table_row_bytes);
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            cs[s][j][0] = load_cached16(rT, off0 + lane_off + (uint32_t)j * step_bytes);
            cs[s][j][1] = load_cached16(rT, off0 + lane_off + (uint32_t)j * step_bytes + 16u);
        }
    }
    template <int TILE> __device__ __forceinline__ void begin_tile(const TileWalk &, int) {}
    __device__ __forceinline__ u32x4 rotate(int s, int j, u32x4 w) const
    {
        return rope_rotate_bf16x8(w, cs[s][j][0], cs[s][j][1]);
    }
    __device__ __forceinline__ void fetch(int s, int j, f32x2 (&e)[4]) const
    {
        e[0] = f32x2{cs[s][j][0].x, cs[s][j][0].y};
        e[1] = f32x2{cs[s][j][0].z, cs[s][j][0].w};
        e[2] = f32x2{cs[s][j][1].x, cs[s][j][1].y};
        e[3] = f32x2{cs[s][j][1].z, cs[s][j][1].w};
    }
    __device__ __forceinline__ u32x4 rotate_with(u32x4 w, const f32x2 (&e)[4]) const
    {
        return u32x4{rope_rotate_pair(w.x, e[0].x, e[0].y), rope_rotate_pair(w.y, e[1].x, e[1].y),
                     rope_rotate_pair(w.z, e[2].x, e[2].y), rope_rotate_pair(w.w, e[3].x, e[3].y)};
    }
};

template <int STEPS, int DEPTH>
struct Rotator<kRope3D, STEPS, DEPTH> {
    const unsigned char *tab;          // the three tables in LDS
    uint32_t base[4], mul_f[4], mul_r[4], mul_c[4];   // entry address of pair q = base + f*mul_f + r*mul_r + c*mul_c
    int rows, cols, rc, frames_m1, row0, rows_per_step;
    float inv_rows, inv_cols;
    int sf, sr, sc;                    // wave-uniform: one stride of the walk as (frames, rows, columns)
    int f[STEPS], r[STEPS], c[STEPS];  // position of the lane's rows of the tile in work

    __device__ __forceinline__ Rotator(const RopeArg &a, int /*t1*/, int d, int row0_, int rows_per_step_, int pair0,
                                       int /*lane_valid*/, const unsigned char *lds_tab)
        : tab(lds_tab), rows(a.r3.rows), cols(a.r3.cols), rc(a.r3.rows * a.r3.cols), frames_m1(a.r3.frames - 1),
          row0(row0_), rows_per_step(rows_per_step_), inv_rows(1.0f / (float)a.r3.rows),
          inv_cols(1.0f / (float)a.r3.cols), sf(0), sr(0), sc(0)
    {
        const Rope3D &R = a.r3;
        const uint32_t off_h = (uint32_t)(R.frames * R.n_t) * 8u, off_w = off_h + (uint32_t)(R.rows * R.n_h) * 8u;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int p = pair0 + q;
            p = p < d / 2 ? p : d / 2 - 1;        // lanes past d (their features are zero) look at a valid entry
            mul_f[q] = mul_r[q] = mul_c[q] = 0u;
            if (p < R.n_t) {
                base[q] = (uint32_t)p * 8u;
                mul_f[q] = (uint32_t)R.n_t * 8u;
            } else if (p < R.n_t + R.n_h) {
                base[q] = off_h + (uint32_t)(p - R.n_t) * 8u;
                mul_r[q] = (uint32_t)R.n_h * 8u;
            } else {
                base[q] = off_w + (uint32_t)(p - R.n_t - R.n_h) * 8u;
                mul_c[q] = (uint32_t)R.n_w * 8u;
            }
        }
    }

    __device__ __forceinline__ void request(int, bool, int) {}

    // Positions of the lane's rows of the i-th tile of the walk; call for i = 0, 1, 2, ... in turn.
    // A walk visits tiles a constant stride apart except where its cyclic order wraps around, so
    // normally every row is the same row of the previous tile plus the stride's (frames, rows,
    // columns), with two carries: ten integer instructions per row and one scalar comparison.
    // Integer divisions (long instruction sequences on this hardware) are left to the first tile
    // and the wrap; there the rows inside the tile are reached from the tile's own position
    // with small carries done in floating point: (x + 0.5) / n is at least 0.5 / n away from
    // an integer and x stays far below 2^20, so the truncated product with the rounded
    // reciprocal is the exact quotient.  A frame index is capped at the last frame: that
    // happens to rows past the last token only (they hold zeros, any entry will do), and a
    // row past the end stays past the end until the walk wraps.
    template <int TILE> __device__ __forceinline__ void begin_tile(const TileWalk &w, int i)
    {
        if (i == 0 || i + w.rot == w.count) {
            if (i == 0) {                                  // one stride as (frames, rows, columns)
                const int stride = w.step * TILE;
                sf = stride / rc;
                const int srem = stride - sf * rc;
                sr = srem / cols;
                sc = srem - sr * cols;
            }
            const int tok0 = w.template token<TILE>(i);
            const int f0 = tok0 / rc, rem = tok0 - f0 * rc, r0 = rem / cols, c0 = rem - r0 * cols;
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
                const int c1 = c0 + row0 + j * rows_per_step;
                const int dr = (int)(((float)c1 + 0.5f) * inv_cols);
                const int r1 = r0 + dr;
                const int df = (int)(((float)r1 + 0.5f) * inv_rows);
                c[j] = c1 - __mul24(dr, cols);
                r[j] = r1 - __mul24(df, rows);
                const int ff = f0 + df;
                f[j] = ff < frames_m1 ? ff : frames_m1;
            }
        } else {
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
                const int cc = c[j] + sc;
                const bool cr = cc >= cols;
                c[j] = cr ? cc - cols : cc;
                const int rr = r[j] + sr + (cr ? 1 : 0);
                const bool cf = rr >= rows;
                r[j] = cf ? rr - rows : rr;
                const int ff = f[j] + sf + (cf ? 1 : 0);
                f[j] = ff < frames_m1 ? ff : frames_m1;
            }
        }
    }

    // The (cos, sin) entries of the lane's four pairs of chunk j: four LDS reads.  Split from the
    // arithmetic so that a caller can issue the reads of a whole tile first and do other work
    // while they are in flight.
    __device__ __forceinline__ void fetch(int /*s*/, int j, f32x2 (&e)[4]) const
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // 24-bit multiplies run at full rate (32-bit ones at a quarter); positions and strides are far below 2^24
            const uint32_t addr = base[q] + __umul24((uint32_t)f[j], mul_f[q]) + __umul24((uint32_t)r[j], mul_r[q]) +
                                  __umul24((uint32_t)c[j], mul_c[q]);
            e[q] = *reinterpret_cast<const f32x2 *>(tab + addr);
        }
    }
    __device__ __forceinline__ u32x4 rotate_with(u32x4 w, const f32x2 (&e)[4]) const
    {
        return u32x4{rope_rotate_pair(w.x, e[0].x, e[0].y), rope_rotate_pair(w.y, e[1].x, e[1].y),
                     rope_rotate_pair(w.z, e[2].x, e[2].y), rope_rotate_pair(w.w, e[3].x, e[3].y)};
    }
    __device__ __forceinline__ u32x4 rotate(int s, int j, u32x4 w) const
    {
        f32x2 e[4];
        fetch(s, j, e);
        return rotate_with(w, e);
    }
};

}  // namespace sv
