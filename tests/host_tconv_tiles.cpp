// Host-side check of the temporal-convolution tile order: compiled with g++ by
// tests/test_host_tile_order.py.  For a range of tile-grid shapes every tile must be
// assigned to exactly one workgroup id of the launch grid, and the eight XCD shares must
// differ by at most one tile.
#include <cstdio>
#include <vector>

#include "../paper_2509_24695_amd/csrc/tconv_tiles.hpp"

int main()
{
    long cases = 0;
    for (int tiles_m = 1; tiles_m <= 300; tiles_m += (tiles_m < 40 ? 1 : 37))
        for (int tiles_n = 1; tiles_n <= 12; ++tiles_n) {
            const long tiles = (long)tiles_m * tiles_n, wgs = sv::tc_grid_size(tiles);
            std::vector<int> hits(tiles, 0);
            long per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (long wg = 0; wg < wgs; ++wg) {
                int tm = -1, tn = -1;
                if (!sv::tc_tile_of(tiles_m, tiles_n, (int)wg, tm, tn)) continue;
                if (tm < 0 || tm >= tiles_m || tn < 0 || tn >= tiles_n) {
                    printf("FAIL %d x %d: workgroup %ld -> tile (%d, %d) out of range\n", tiles_m, tiles_n, wg, tm, tn);
                    return 1;
                }
                ++hits[(long)tm * tiles_n + tn];
                ++per_xcd[wg & 7];
            }
            for (long t = 0; t < tiles; ++t)
                if (hits[t] != 1) {
                    printf("FAIL %d x %d: tile %ld assigned %d times\n", tiles_m, tiles_n, t, hits[t]);
                    return 1;
                }
            long lo = per_xcd[0], hi = per_xcd[0];
            for (int e = 1; e < 8; ++e) { lo = per_xcd[e] < lo ? per_xcd[e] : lo; hi = per_xcd[e] > hi ? per_xcd[e] : hi; }
            if (hi - lo > 1) {
                printf("FAIL %d x %d: XCD shares from %ld to %ld tiles\n", tiles_m, tiles_n, lo, hi);
                return 1;
            }
            ++cases;
        }
    printf("OK %ld tile grids\n", cases);
    return 0;
}
