// Grouped launch: several independent products of different shapes (one input type, one B
// storage, one kernel variant) share one grid.  The paper names grouped GEMM only as a further
// multiplier of a tuning search (Sections II-B and V-C); for the analytical selector it is one
// more evaluation of the model over the groups' tiles.
//
// The tiles of group g occupy the logical workgroup ids [tile_start[g], tile_start[g+1]) of
// the launch, each group rasterised in its own grouped order.  The kernel finds its group by a
// binary search over a table of fixed-size records in device memory; the same records and the
// same search run on the host (plan construction, validation, tests).
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
    int tile_start;       // first logical workgroup id of the group
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

// The group that owns logical id l in [0, total tiles): the last g with tile_start[g] <= l
// (tile_start[0] is 0; empty groups share their successor's start and are never returned for
// an id inside the grid unless they are trailing, which the `<=` rule also skips).
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
