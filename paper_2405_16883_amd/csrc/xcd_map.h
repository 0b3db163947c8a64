// Which column tile and which unit of row work a workgroup owns, and how many workgroups a launch needs.
// Plain integer arithmetic with no HIP dependency, so that the host tests can compile and check it on the CPU.
//
// Default (xcd_slices == 0): tile-major (all row work of column tile 0, then tile 1, ...).
// XCD-sliced (xcd_slices != 0): workgroups are dealt to the 8 XCDs round-robin by index, and each XCD has its own
// L2.  Every XCD is therefore given its own narrow column slices of B, one after the other, so that the slice it is
// gathering from stays resident in that XCD's L2.  The slices are taken in rounds: first whole rounds of 8 slices,
// one per XCD; then the remaining r < 8 slices in groups of 4, 2 and 1 (the binary digits of r), a group of s slices
// being shared by all 8 XCDs, 8/s XCDs per slice, which split that slice's row work between them.  Every round keeps
// all XCDs equally busy whatever the number of slices.  The mapping only steers locality; any assignment of workgroups
// to XCDs gives the same result.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define SCORCH_HOST_DEVICE __host__ __device__
#else
#define SCORCH_HOST_DEVICE
#endif

namespace scorch {

constexpr int kXcds = 8;  // accelerator dies, each with its own L2; workgroups are dealt to them round-robin

// Workgroup `index` of the launch owns unit `b` (< per_tile) of column tile `ct`; false: the workgroup has no work
// (padding of a shared round).
SCORCH_HOST_DEVICE inline bool tile_of_index(uint32_t index, int32_t xcd_slices, int32_t ncoltiles, uint32_t per_tile,
                                             uint32_t &ct, uint32_t &b) {
    if (xcd_slices == 0) {
        ct = index / per_tile;
        b = index - ct * per_tile;
        return true;
    }
    const uint32_t xcd = index & (kXcds - 1);
    uint32_t q = index / kXcds;
    const uint32_t rounds = (uint32_t)ncoltiles / kXcds, rest = (uint32_t)ncoltiles % kXcds;
    if (q < rounds * per_tile) {
        const uint32_t round = q / per_tile;
        b = q - round * per_tile;
        ct = xcd + kXcds * round;
        return true;
    }
    q -= rounds * per_tile;
    uint32_t base = rounds * kXcds;
    for (uint32_t s = kXcds / 2; s >= 1; s >>= 1) {
        if (rest & s) {
            const uint32_t share = kXcds / s;  // XCDs per slice of this group
            const uint32_t nq = (per_tile + share - 1) / share;
            if (q < nq) {
                ct = base + xcd % s;
                b = q * share + xcd / s;
                return b < per_tile;
            }
            q -= nq;
            base += s;
        }
    }
    return false;
}

// Number of workgroups for `per_tile` units of row work per column tile.
inline int64_t xcd_grid_size(int32_t xcd_slices, int32_t ncoltiles, int64_t per_tile) {
    if (xcd_slices == 0) return per_tile * ncoltiles;
    int64_t q = (int64_t)(ncoltiles / kXcds) * per_tile;
    const int rest = ncoltiles % kXcds;
    for (int s = kXcds / 2; s >= 1; s >>= 1)
        if (rest & s) q += (per_tile * s + kXcds - 1) / kXcds;
    return q * kXcds;
}

}  // namespace scorch
