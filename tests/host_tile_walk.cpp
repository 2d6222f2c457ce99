// Host-side check of the token-tile walk of the attention kernels: compiled with g++ by
// tests/test_host_tile_order.py.  For many (token range, chunk count, head) combinations the walks of
// all waves of all workgroups of a head together must visit every tile of the range exactly once,
// stay inside the range, and report kOutOfRange past a wave's share.  Also: the slices in which the
// workgroups of a head fold its state must partition the state's 8-byte units, and the shares of the
// one-launch block step must be a permutation of the workgroups in every head.
#include <cstdio>
#include <vector>

#include "../paper_2509_24695_amd/csrc/tile_walk.hpp"

template <int TILE>
static bool check(int t0, int t1, int C, int waves, bool wave_private, int bh)
{
    const int n_tiles = (t1 - t0 + TILE - 1) / TILE;
    std::vector<int> hits(n_tiles, 0);
    for (int c = 0; c < C; ++c)
        for (int w = 0; w < (wave_private ? waves : 1); ++w) {
            const sv::TileWalk walk = wave_private ? sv::TileWalk(t0, waves * c + w, waves * C, n_tiles, bh)
                                                   : sv::TileWalk(t0, c, C, n_tiles, bh);
            for (int i = 0; i < walk.count; ++i) {
                const int tok = walk.token<TILE>(i);
                if (tok < t0 || tok >= t1 || (tok - t0) % TILE != 0) return false;
                if (walk.offset<TILE>(i, 128u) != (uint32_t)tok * 128u) return false;
                ++hits[(tok - t0) / TILE];
            }
            for (int i = walk.count; i < walk.count + 9; ++i)
                if (walk.offset<TILE>(i, 128u) != sv::kOutOfRange) return false;
        }
    for (int h : hits)
        if (h != 1) return false;
    return true;
}

static bool check_slices(int d, int C)
{
    const int units = d * d / 2 + d / 2;
    std::vector<int> hits(units, 0);
    for (int c = 0; c < C; ++c) {
        const sv::StateSlice sl(c, C, d);
        if (sl.units != units || sl.s_units != d * d / 2 || sl.lo < 0 || sl.hi > units || sl.lo > sl.hi) return false;
        for (int v = sl.lo; v < sl.hi; ++v) ++hits[v];
    }
    for (int h : hits)
        if (h != 1) return false;
    return true;
}

static bool check_shares(int C, int bh)
{
    std::vector<int> hits(C, 0);
    for (int c = 0; c < C; ++c) {
        const int s = sv::block_step_share(c, bh, C);
        if (s < 0 || s >= C) return false;
        ++hits[s];
    }
    for (int h : hits)
        if (h != 1) return false;
    return true;
}

int main()
{
    long cases = 0;
    for (int d : {2, 8, 32, 64, 112, 128})
        for (int C = 1; C <= 64; ++C)
            if (!check_slices(d, C)) {
                printf("FAIL slices d=%d C=%d\n", d, C);
                return 1;
            }
    for (int C = 1; C <= 32; ++C)
        for (int bh = 0; bh < 700; bh += 7)
            if (!check_shares(C, bh)) {
                printf("FAIL shares C=%d bh=%d\n", C, bh);
                return 1;
            }
    const int ranges[][2] = {{0, 1}, {0, 15}, {0, 16}, {0, 33}, {5, 5 + 1000}, {64, 64 + 4680}, {0, 32760}, {17, 17 + 12345}};
    for (const auto &r : ranges)
        for (int C = 1; C <= 32; C += (C < 9 ? 1 : 5))
            for (int bh = 0; bh < 40; bh += 3) {
                bool ok = check<32>(r[0], r[1], C, 4, true, bh) && check<16>(r[0], r[1], C, 4, true, bh) &&
                          check<32>(r[0], r[1], C, 4, false, bh) && check<64>(r[0], r[1], C, 4, false, bh);
                if (!ok) {
                    printf("FAIL range [%d, %d) C=%d bh=%d\n", r[0], r[1], C, bh);
                    return 1;
                }
                cases += 4;
            }
    printf("OK %ld walks\n", cases);
    return 0;
}
