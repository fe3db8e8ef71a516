// Host-only fuzz driver for the selector-side entry points of the C ABI; built with the
// address and undefined-behaviour sanitizers by tests/test_host_sanitizers.py (no GPU code
// involved).  Random shapes, all dtypes, both storages of B, batches; every enumerated cfg
// goes through gemm_predict and gemm_workspace_bytes, every Stream-K cfg through the plan
// functions with a check that the workers' segments cover each K slab exactly once.
#include "gemm.h"
#include <cstdio>
#include <cstdlib>
#include <vector>

static unsigned s = 1;
static long rnd(long n) { s = s * 1664525u + 1013904223u; return (long)((s >> 8) % (unsigned long)n); }

static int check_stream_k(const gemm_cfg &c)
{
    int32_t plan[4];
    if (gemm_stream_k_plan(&c, plan) != GEMM_OK)
        return 10;
    const int G = plan[0], sk = plan[1], S = plan[3];
    std::vector<int> cover((size_t)sk * S, 0);
    for (int g = 0; g < G; ++g) {
        gemm_sk_segment seg[2];
        const int n = gemm_stream_k_segments(&c, g, seg);
        if (n < 1 || n > 2)
            return 11;
        for (int i = 0; i < n; ++i) {
            if (seg[i].sk_tile < 0 || seg[i].sk_tile >= sk || seg[i].slab0 < 0 || seg[i].count < 1 ||
                seg[i].slab0 + seg[i].count > S)
                return 12;
            for (int k = 0; k < seg[i].count; ++k)
                ++cover[(size_t)seg[i].sk_tile * S + seg[i].slab0 + k];
        }
    }
    for (int v : cover)
        if (v != 1)
            return 13;
    for (int j = 0; j < sk; j += 1 + sk / 16) {
        int32_t out3[3];
        if (gemm_stream_k_contributors(&c, j, out3) != GEMM_OK || out3[0] > out3[1] || out3[1] >= G)
            return 14;
    }
    gemm_sk_segment seg[2];
    if (gemm_stream_k_segments(&c, G, seg) != GEMM_ERR_INDEX || gemm_stream_k_contributors(&c, sk, plan) != GEMM_ERR_INDEX)
        return 15;
    return 0;
}

int main()
{
    gemm_cfg c;
    gemm_prediction p;
    long acc = 0, n_sk = 0;
    for (int it = 0; it < 1500; ++it) {
        // every fourth shape has N and K that are not whole 16-byte chunks
        const bool ragged = it % 4 == 3;
        const long M = 1 + rnd(16384), N = ragged ? 1 + rnd(16384) : 16 * (1 + rnd(1024)),
                   K = ragged ? 1 + rnd(16384) : 16 * (1 + rnd(1024));
        const int dt = it % 3, bl = (it / 3) & 1;
        const long batch = (it % 5 == 0) ? 1 + rnd(64) : 1;
        if (gemm_select_batched(M, N, K, batch, dt, bl, &c) != GEMM_OK) {
            printf("select failed %ld %ld %ld\n", M, N, K);
            return 1;
        }
        if (gemm_predict(&c, &p) != GEMM_OK || !(p.total_us > 0))
            return 2;
        acc += c.kernel_id + (long)gemm_workspace_bytes(&c) % 7;
        for (int i = (int)rnd(5); i < gemm_cfg_count(dt); i += 5) {
            gemm_cfg d;
            const int rc = gemm_cfg_at_batched(i, M, N, K, batch, dt, bl, &d);
            if (rc == GEMM_ERR_CFG_ILLEGAL)
                continue;
            if (rc != GEMM_OK || gemm_predict(&d, &p) != GEMM_OK)
                return 3;
            if (d.stream_k) {
                if (batch != 1)
                    return 4;
                ++n_sk;
                const int e = check_stream_k(d);
                if (e)
                    return e;
            }
        }
    }
    // grouped selection and plans over random group lists (with empty groups); every record's tile
    // range must tile [0, total) in order
    for (int it = 0; it < 200; ++it) {
        const int n = 1 + (int)rnd(it % 10 == 0 ? 4096 : 40), dt = it % 3, bl = (it / 3) & 1;
        static gemm_problem probs[4096];
        static gemm_group_rec table[4096];
        const long N = 16 * (1 + rnd(256)), K = 16 * (1 + rnd(256));
        bool any = false;
        for (int i = 0; i < n; ++i) {
            const long M = rnd(4) == 0 ? 0 : 1 + rnd(700);
            any = any || M > 0;
            probs[i].M = M;
            probs[i].N = (it & 1) ? N : 16 * (1 + rnd(256));
            probs[i].K = (it & 1) ? K : 16 * (1 + rnd(256));
            probs[i].lda = probs[i].K;
            probs[i].ldb = bl ? probs[i].K : probs[i].N;
            probs[i].ldc = probs[i].N;
            probs[i].A = probs[i].B = (const void *)(uintptr_t)(0x1000 * (i + 1));
            probs[i].C = (void *)(uintptr_t)(0x1000 * (i + 1));
        }
        const int rc = gemm_select_grouped(n, probs, dt, bl, &c);
        if (!any) {
            if (rc != GEMM_ERR_SHAPE)
                return 20;
            continue;
        }
        if (rc != GEMM_OK || c.groups != n || !(c.predicted_us > 0))
            return 21;
        int64_t total = 0, start = 0;
        if (gemm_grouped_plan(&c, n, probs, table, &total) != GEMM_OK)
            return 22;
        gemm_hw hwd;
        gemm_hw_get(&hwd);
        const int X = hwd.n_xcd;
        int64_t tiles = 0;
        for (int i = 0; i < n; ++i) {
            if (table[i].tile_start != start || table[i].group_m < 1 || (i && table[i].K > table[i - 1].K))
                return 23;
            const int64_t t = (int64_t)table[i].tiles_m * table[i].tiles_n;
            start += (t + X - 1) / X;
            tiles += t;
        }
        if (start * X != total || total < 1)
            return 24;
        // sampled workgroups land on a tile inside their record or on an idle slot
        int64_t busy = 0;
        const int64_t step = total > 4000 ? total / 2000 : 1;
        for (int64_t w = 0; w < total; w += step) {
            int32_t o[3];
            if (gemm_grouped_locate(&c, n, table, w, o) != GEMM_OK)
                return 26;
            if (o[0] >= 0) {
                if (o[0] >= n || o[1] < 0 || o[1] >= table[o[0]].tiles_m || o[2] < 0 || o[2] >= table[o[0]].tiles_n)
                    return 27;
                ++busy;
            }
        }
        if (step == 1 && busy != tiles)
            return 28;
        int32_t o[3];
        if (gemm_grouped_locate(&c, n, table, total, o) != GEMM_ERR_INDEX)
            return 29;
        gemm_cfg d;
        const int v = (int)rnd(gemm_variant_count(dt));
        const int rc2 = gemm_cfg_at_grouped(v, n, probs, dt, bl, &d);
        if (rc2 != GEMM_OK && rc2 != GEMM_ERR_CFG_ILLEGAL)
            return 25;
        acc += c.kernel_id;
    }
    // every preset installs, selects and resets
    for (int id = 0; id < 2; ++id) {
        gemm_hw h;
        if (gemm_hw_preset(id, &h) != GEMM_OK || gemm_hw_set(&h) != GEMM_OK)
            return 5;
        if (gemm_select(4096 + 256 * id, 4096, 4096, 0, &c) != GEMM_OK)
            return 6;
        gemm_hw_reset();
    }
    // shapes at the documented limits: every answer is a status, and an accepted cfg predicts and plans
    {
        const long big = 1L << 30, dims[][3] = {{big, big, 1}, {big, 1, big}, {1, big, big}, {big, big, big}, {big, 16, 16},
                                                {1, 1, 1}, {1, big, 1}, {big + 1, 16, 16}};
        for (const auto &d : dims)
            for (int dt = 0; dt < 3; ++dt)
                for (int bl = 0; bl < 2; ++bl) {
                    const int rc = gemm_select(d[0], d[1], d[2], dt, &c);
                    if (d[0] > big ? rc != GEMM_ERR_SHAPE : (rc != GEMM_OK && rc != GEMM_ERR_SHAPE))
                        return 30;
                    if (rc == GEMM_OK && (gemm_predict(&c, &p) != GEMM_OK || !(p.total_us > 0)))
                        return 31;
                    for (int i = 0; i < gemm_cfg_count(dt); i += 7) {
                        gemm_cfg e;
                        const int r2 = gemm_cfg_at_batched(i, d[0], d[1], d[2], 1, dt, bl, &e);
                        if (r2 == GEMM_OK && e.stream_k && check_stream_k(e))
                            return 32;
                        if (r2 == GEMM_OK)
                            acc += (long)(gemm_workspace_bytes(&e) % 3);
                    }
                }
        // a group whose tile count does not fit 31 bits is refused by the plan, not wrapped
        gemm_problem one{};
        one.M = one.N = big;
        one.K = 64;
        one.lda = 64;
        one.ldb = one.ldc = big;
        one.A = one.B = (const void *)(uintptr_t)0x1000;
        one.C = (void *)(uintptr_t)0x1000;
        gemm_group_rec rec;
        int64_t total = 0;
        const int rc = gemm_select_grouped(1, &one, 0, 0, &c);
        if (rc == GEMM_OK && gemm_grouped_plan(&c, 1, &one, &rec, &total) == GEMM_OK)
            return 33;
    }
    // device descriptions: counts beyond the documented bounds are refused; a highly composite CU
    // count inside them (48 divisors) selects and plans without overrunning the factor search
    {
        gemm_hw h0, hx;
        gemm_hw_get(&h0);
        hx = h0;
        hx.n_cu = 55440;
        if (gemm_hw_set(&hx) != GEMM_ERR_SHAPE)
            return 34;
        hx = h0;
        hx.simd_per_cu = 65;
        if (gemm_hw_set(&hx) != GEMM_ERR_SHAPE)
            return 35;
        hx = h0;
        hx.n_cu = 2520;
        hx.n_xcd = 8;
        if (gemm_hw_set(&hx) != GEMM_OK)
            return 36;
        for (int it = 0; it < 60; ++it) {
            const long M = 1 + rnd(8192), N = 1 + rnd(8192), K = 1 + rnd(8192);
            if (gemm_select(M, N, K, it % 3, &c) != GEMM_OK || gemm_predict(&c, &p) != GEMM_OK)
                return 37;
            for (int i = 0; i < gemm_cfg_count(it % 3); i += 3) {
                gemm_cfg e;
                if (gemm_cfg_at(i, M, N, K, it % 3, &e) == GEMM_OK && e.stream_k && check_stream_k(e))
                    return 38;
            }
        }
        gemm_hw_reset();
    }
    gemm_hw h;
    if (gemm_hw_preset(9, &h) != GEMM_ERR_INDEX || gemm_select_batched(64, 64, 64, 0, 0, 0, &c) != GEMM_ERR_SHAPE)
        return 7;
    printf("ok %ld stream-k cfgs %ld\n", acc, n_sk);
    return n_sk > 100 ? 0 : 8;
}
