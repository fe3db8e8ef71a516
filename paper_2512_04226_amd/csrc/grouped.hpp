// Grouped launch: several independent products of different shapes (one input type, one B
// storage, one kernel variant) share one grid.  The paper names grouped GEMM only as a further
// multiplier of a tuning search (Sections II-B and V-C); for the analytical selector it is one
// more evaluation of the model over the groups' tiles.
//
// Hardware deals consecutive workgroup ids round-robin to the X XCDs, and an XCD works through
// its ids in order.  Workgroup id p is therefore slot q = p / X of XCD x = p % X, and every
// group owns the same slot range [slot_start[g], slot_start[g] + ceil(T_g / X)) on every XCD:
// XCD x computes the x-th of X contiguous chunks of the group's T_g tiles (in the group's own
// grouped rasterisation order), exactly as in a launch of that group alone.  Each group is so
// spread over all L2s -- groups with long K loops do not pile up on one XCD -- and a group's
// last slot is idle on the XCDs whose chunk is one tile shorter (the workgroup exits at once).
// With the XCD renumbering switched off X is 1: slots are tiles.
// The kernel finds its group by a binary search over a table of fixed-size records in device
// memory; the same records and the same arithmetic run on the host (plan, validation, tests).
#pragma once
#include <stdint.h>

#include "stream_k.hpp"

namespace g355 {

struct GroupRec {
    const void *A;
    const void *B;
    void *C;
    int M, N, K;          // M may be 0: an empty group owns no tiles
    int lda, ldb, ldc;    // elements
    int tiles_m, tiles_n;
    int tile_start;       // first per-XCD slot of the group: sum of ceil(T / X) over the records before it
    int group_m;          // band height of the group's rasterisation
};
static_assert(sizeof(GroupRec) == 64, "one record is 64 bytes");

// A value every lane of the wave holds alike, kept in a scalar register on the device.
G355_HD inline int uniform_i32(int x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_readfirstlane(x);
#else
    return x;
#endif
}

template <class P>
G355_HD inline P uniform_ptr(P p)
{
    const uint64_t u = (uint64_t)p;
    const uint32_t lo = (uint32_t)uniform_i32((int)(uint32_t)u), hi = (uint32_t)uniform_i32((int)(uint32_t)(u >> 32));
    return (P)(((uint64_t)hi << 32) | lo);
}

// Slots a group of `tiles` tiles takes on each of X XCDs.
G355_HD inline int group_slots(int tiles, int X) { return (tiles + X - 1) / X; }

// Tile of a group (index in its rasterisation order) computed in slot j of XCD x, or -1 when
// that slot is idle: XCD x owns the x-th contiguous chunk, the first tiles % X chunks one longer.
G355_HD inline int group_tile(int tiles, int X, int x, int j)
{
    const int per = tiles / X, rem = tiles % X;
    if (j >= per + (x < rem ? 1 : 0))
        return -1;
    return x * per + (x < rem ? x : rem) + j;
}

// The group that owns slot l in [0, total slots): the last g with tile_start[g] <= l
// (tile_start[0] is 0; empty groups share their successor's start and are never returned for
// a slot inside the grid unless they are trailing, which the `<=` rule also skips).
G355_HD inline int group_of(const GroupRec *tab, int n, int l)
{
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (uniform_i32(tab[mid].tile_start) <= l)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

}  // namespace g355
