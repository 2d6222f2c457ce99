// Tile order of the temporal-convolution kernel: which tile a workgroup id works on.
// Plain C++ (no device code), shared by the kernel, the launcher and a host-side test.
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

constexpr int kTcGroupM = 4;   // token tiles per group of the tile order

// Workgroups a grid needs for `tiles` tiles: eight XCD shares, each as long as the longest.
SV_HOST_DEVICE inline int64_t tc_grid_size(int64_t tiles) { return 8 * ((tiles + 7) / 8); }

// Workgroup id -> tile (token tile tm < tiles_m, channel tile tn < tiles_n); false if the id has no
// tile.  Tiles are ordered in groups of kTcGroupM token tiles, token tile fastest inside a group;
// consecutive workgroup ids go to the eight XCDs in turn, each with its own L2, so XCD e takes the
// e-th eighth of that order: the workgroups that run on one XCD at a time share a few token tiles
// and W's current K-slice, and all XCDs get the same number of tiles (to within one) however few
// there are.
SV_HOST_DEVICE inline bool tc_tile_of(int tiles_m, int tiles_n, int wg, int &tm, int &tn)
{
    const int64_t tiles = (int64_t)tiles_m * tiles_n;
    const int xcd = wg & 7, seq = wg >> 3;
    const int64_t begin = (xcd * tiles) >> 3, end = ((xcd + 1) * tiles) >> 3;
    const int64_t t = begin + seq;
    if (t >= end) return false;
    const int per_group = kTcGroupM * tiles_n, g = (int)(t / per_group), in = (int)(t - (int64_t)g * per_group);
    const int left = tiles_m - g * kTcGroupM, rows = left < kTcGroupM ? left : kTcGroupM;   // token tiles in this group
    tn = in / rows;
    tm = g * kTcGroupM + (in - tn * rows);
    return true;
}

}  // namespace sv
