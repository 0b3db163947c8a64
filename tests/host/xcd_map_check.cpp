// CPU check of the workgroup -> (column tile, unit of row work) mapping used by the XCD-sliced launches.
// For every (number of column tiles, units per tile) in a range it verifies that
//   * the launch covers every (tile, unit) pair exactly once and nothing outside the ranges,
//   * the grid is a multiple of 8 workgroups (whole rounds over the XCDs) in the sliced mode,
//   * in the sliced mode a tile of a whole round is served by a single XCD (workgroup index mod 8), and a tile of
//     a shared round by exactly 8/s XCDs, s being the size of its group (4, 2 or 1),
//   * the XCDs' shares of the work differ by at most one unit per shared group.
// Prints "ok <cases>" or the first failure.
#include <algorithm>
#include <cstdio>
#include <set>
#include <vector>

#include "xcd_map.h"

using namespace scorch;

int main() {
    long cases = 0;
    for (int mode = 0; mode <= 1; ++mode)
        for (int nt = 1; nt <= 41; ++nt)
            for (uint32_t per : {1u, 2u, 3u, 5u, 7u, 8u, 9u, 13u, 64u, 257u}) {
                const int64_t grid = xcd_grid_size(mode, nt, per);
                if (mode && grid % kXcds) { std::printf("grid %lld not a multiple of 8 (nt=%d per=%u)\n", (long long)grid, nt, per); return 1; }
                std::vector<int> seen((size_t)nt * per, 0);
                std::vector<std::set<int>> xcds_of_tile(nt);
                std::vector<long> work(kXcds, 0);
                for (int64_t i = 0; i < grid; ++i) {
                    uint32_t ct = ~0u, b = ~0u;
                    if (!tile_of_index((uint32_t)i, mode, nt, per, ct, b)) {
                        if (!mode) { std::printf("idle workgroup in tile-major mode\n"); return 1; }
                        continue;
                    }
                    if (ct >= (uint32_t)nt || b >= per) { std::printf("out of range: nt=%d per=%u i=%lld -> (%u,%u)\n", nt, per, (long long)i, ct, b); return 1; }
                    if (seen[(size_t)ct * per + b]++) { std::printf("pair served twice: nt=%d per=%u (%u,%u)\n", nt, per, ct, b); return 1; }
                    xcds_of_tile[ct].insert((int)(i % kXcds));
                    work[i % kXcds]++;
                }
                for (size_t x = 0; x < seen.size(); ++x)
                    if (!seen[x]) { std::printf("pair never served: mode=%d nt=%d per=%u tile=%zu unit=%zu\n", mode, nt, per, x / per, x % per); return 1; }
                if (mode) {
                    const int rounds = nt / kXcds, rest = nt % kXcds;
                    int base = rounds * kXcds;
                    for (int t = 0; t < base; ++t)
                        if (xcds_of_tile[t].size() != 1 || *xcds_of_tile[t].begin() != t % kXcds) { std::printf("tile %d of a whole round not on its XCD (nt=%d per=%u)\n", t, nt, per); return 1; }
                    int groups = 0;
                    for (int s = kXcds / 2; s >= 1; s >>= 1)
                        if (rest & s) {
                            ++groups;
                            for (int t = base; t < base + s; ++t) {
                                const size_t want = (size_t)std::min<uint32_t>(kXcds / s, per);
                                if (xcds_of_tile[t].size() != want) { std::printf("tile %d shared by %zu XCDs, expected %zu (nt=%d per=%u)\n", t, xcds_of_tile[t].size(), want, nt, per); return 1; }
                            }
                            base += s;
                        }
                    long lo = work[0], hi = work[0];
                    for (long w : work) { lo = w < lo ? w : lo; hi = w > hi ? w : hi; }
                    if (hi - lo > groups) { std::printf("XCD loads differ by %ld with %d shared groups (nt=%d per=%u)\n", hi - lo, groups, nt, per); return 1; }
                }
                ++cases;
            }
    std::printf("ok %ld\n", cases);
    return 0;
}
