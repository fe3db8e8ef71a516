// Stream-K work split (the wave-quantisation remedy the paper's kernels use, Section V-E),
// in the hybrid form: whole waves of output tiles stay data-parallel, and the tiles of the
// last, partial wave are cut along K into equal iteration ranges, one per worker.
//
//   tiles       output tiles of the problem, in the rasterisation's logical order
//   workers     G: workgroups that share the stream-K tiles (one per workgroup slot of the device)
//   sk_tiles    tiles % G  (the partial wave), the LAST sk_tiles logical tiles
//   dp_tiles    tiles - sk_tiles, one workgroup each
//   slabs       S: K_T slabs per tile
//   iters       sk_tiles * S, numbered tile-major: iteration x is slab x % S of stream-K tile x / S
//
// Worker g owns iterations [g*iters/G, (g+1)*iters/G) (integer floors).  Because
// sk_tiles < G, a range is at most S long and touches at most two tiles: at most two
// segments per worker.  A segment that covers its whole tile is written to C directly;
// every other segment leaves an fp32 partial tile in workspace slot 2*g + (segment number),
// and a second kernel sums a tile's partials in worker order.  No workgroup ever waits for
// another one.
//
// The same functions run on the host (validation, tests) and on the device.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define G355_HD __host__ __device__
#else
#define G355_HD
#endif

namespace g355 {

// Logical tile id t -> tile coordinates: ids run column-major through bands of group_m tile
// rows (the rasterisation order of the kernel; stream-K tiles are the last ids of it).
G355_HD inline void logical_tile(int tiles_m, int tiles_n, int group_m, int t, int &tm, int &tn)
{
    const int band_sz = group_m * tiles_n;
    const int band = t / band_sz;
    const int first_m = band * group_m;
    const int rows = (tiles_m - first_m < group_m) ? (tiles_m - first_m) : group_m;
    const int r = t - band * band_sz;
    tm = first_m + r % rows;
    tn = r / rows;
}

struct SkPlan {
    int workers;    // G >= 1
    int sk_tiles;   // 1 .. G-1 (or all tiles when there are fewer than G)
    int dp_tiles;
    int slabs;      // S >= 1
    int64_t iters;  // sk_tiles * S >= G, so that no worker is idle
};

struct SkSegment {
    int tile;       // stream-K tile index in [0, sk_tiles)
    int slab0;      // first slab of the tile this segment covers
    int count;      // slabs covered, >= 1
    int complete;   // 1: the segment is the whole tile
};

G355_HD inline int64_t sk_first_iter(const SkPlan &p, int g) { return (int64_t)g * p.iters / p.workers; }

// The worker whose range contains iteration x: the largest g with floor(g*iters/G) <= x.
G355_HD inline int sk_owner(const SkPlan &p, int64_t x)
{
    int64_t g = ((x + 1) * p.workers - 1) / p.iters;
    if (g > p.workers - 1)
        g = p.workers - 1;
    return (int)g;
}

// Segments of worker g (0, 1 or 2); returns their number.
G355_HD inline int sk_segments(const SkPlan &p, int g, SkSegment seg[2])
{
    const int64_t b = sk_first_iter(p, g), e = sk_first_iter(p, g + 1);
    if (e <= b)
        return 0;
    const int64_t S = p.slabs;
    const int64_t t = b / S;
    const int64_t cut = (t + 1) * S;
    const int64_t e0 = e < cut ? e : cut;
    seg[0].tile = (int)t;
    seg[0].slab0 = (int)(b - t * S);
    seg[0].count = (int)(e0 - b);
    seg[0].complete = (seg[0].count == p.slabs);
    if (e <= cut)
        return 1;
    seg[1].tile = (int)(t + 1);
    seg[1].slab0 = 0;
    seg[1].count = (int)(e - cut);
    seg[1].complete = (seg[1].count == p.slabs);
    return 2;
}

// Contributors of stream-K tile j: workers g_first .. g_last, in that order.  When one
// worker covers the whole tile (g_first == g_last) there is nothing to sum.  Worker g's
// partial for tile j sits in slot 2*g + sk_slot_of(p, g, j).
G355_HD inline void sk_contributors(const SkPlan &p, int j, int *g_first, int *g_last)
{
    *g_first = sk_owner(p, (int64_t)j * p.slabs);
    *g_last = sk_owner(p, (int64_t)(j + 1) * p.slabs - 1);
}
G355_HD inline int sk_slot_of(const SkPlan &p, int g, int j) { return (sk_first_iter(p, g) / p.slabs == j) ? 0 : 1; }

// Plan for a problem; returns false when stream-K does not apply (no partial wave, or fewer
// iterations than workers).
G355_HD inline bool sk_make_plan(int64_t tiles, int workers, int64_t slabs, SkPlan *p)
{
    if (workers < 1 || tiles < 1 || slabs < 1 || workers > 65535)
        return false;
    const int64_t sk = tiles % workers;
    if (sk == 0)
        return false;
    if (sk * slabs < workers || sk * slabs >= ((int64_t)1 << 31) || tiles >= ((int64_t)1 << 31))
        return false;
    p->workers = workers;
    p->sk_tiles = (int)sk;
    p->dp_tiles = (int)(tiles - sk);
    p->slabs = (int)slabs;
    p->iters = sk * slabs;
    return true;
}

}  // namespace g355
