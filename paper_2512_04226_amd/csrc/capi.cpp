// Host-only entry points of the C ABI: selection, enumeration, prediction, hardware
// descriptor.  Nothing here touches the GPU.
#include <algorithm>
#include <cstring>

#include "../../include/gemm.h"
#include "model.hpp"
#include "grouped.hpp"
#include "stream_k.hpp"

using namespace g355;

namespace g355 {
int check_problem(int64_t M, int64_t N, int64_t K, int dtype)
{
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3 && dtype != GEMM_FP16)
        return GEMM_ERR_DTYPE;
    if (M < 1 || N < 1 || K < 1)
        return GEMM_ERR_SHAPE;
    const int64_t lim = (int64_t)1 << 30;
    if (M > lim || N > lim || K > lim)
        return GEMM_ERR_SHAPE;
    return GEMM_OK;   // N and K need not be whole 16-byte chunks: such shapes run the trimming instantiation
}

// The stream-K plan a cfg describes, or false when its fields do not make one.
bool cfg_stream_k_plan(const gemm_cfg *cfg, SkPlan *p)
{
    if (cfg->stream_k != 1 || cfg->split_k != 1 || cfg->block_m < 1 || cfg->block_n < 1 || cfg->block_k < 1 ||
        cfg->group_m < 1 || check_problem(cfg->M, cfg->N, cfg->K, cfg->dtype))
        return false;
    const int64_t tiles_m = (cfg->M + cfg->block_m - 1) / cfg->block_m, tiles_n = (cfg->N + cfg->block_n - 1) / cfg->block_n;
    return sk_make_plan(tiles_m * tiles_n, cfg->sk_workers, (cfg->K + cfg->block_k - 1) / cfg->block_k, p);
}

int check_grouped_cfg(const gemm_cfg *cfg, int n_groups)
{
    if (cfg->abi_version != GEMM_ABI_VERSION)
        return GEMM_ERR_ABI;
    if (n_groups < 1 || n_groups > kMaxGroups)
        return GEMM_ERR_SHAPE;
    if (cfg->dtype != GEMM_BF16 && cfg->dtype != GEMM_FP8_E4M3 && cfg->dtype != GEMM_FP16)
        return GEMM_ERR_DTYPE;
    if (cfg->groups != n_groups || cfg->kernel_id < 0 || cfg->kernel_id >= variant_count(cfg->dtype))
        return GEMM_ERR_CFG_ILLEGAL;
    const Variant &v = variant_at(cfg->dtype, cfg->kernel_id);
    if (cfg->block_m != v.block_m || cfg->block_n != v.block_n || cfg->block_k != v.block_k ||
        cfg->waves_m != v.waves_m || cfg->waves_n != v.waves_n || cfg->mfma != v.mfma || cfg->stages != v.stages)
        return GEMM_ERR_CFG_ILLEGAL;
    if (cfg->split_k != 1 || cfg->stream_k || cfg->batch != 1 || cfg->b_layout > 1)
        return GEMM_ERR_CFG_ILLEGAL;
    return GEMM_OK;
}

int grouped_xcds(const gemm_cfg *cfg) { return cfg->xcd_remap ? hw_current().n_xcd : 1; }

int check_group_rec(const gemm_cfg *cfg, const gemm_group_rec *r, int64_t slot_start)
{
    const Variant &v = variant_at(cfg->dtype, cfg->kernel_id);
    if (r->tile_start != slot_start || r->group_m < 1)
        return GEMM_ERR_CFG_ILLEGAL;
    if (r->M == 0)
        return r->tiles_m == 0 ? GEMM_OK : GEMM_ERR_CFG_ILLEGAL;   // owns no tile: nothing else is read
    if (r->M < 0)
        return GEMM_ERR_SHAPE;
    const int rc = check_problem(r->M, r->N, r->K, cfg->dtype);
    if (rc)
        return rc;
    if (!variant_legal(hw_current(), v, cfg->dtype, r->M, r->N, r->K, 1, 0, 1))
        return GEMM_ERR_CFG_ILLEGAL;
    if (r->tiles_m != (r->M + v.block_m - 1) / v.block_m || r->tiles_n != (r->N + v.block_n - 1) / v.block_n)
        return GEMM_ERR_CFG_ILLEGAL;
    if (!r->A || !r->B || !r->C)
        return GEMM_ERR_NULL;
    if (r->lda < r->K || r->ldb < (cfg->b_layout ? r->K : r->N) || r->ldc < r->N)
        return GEMM_ERR_SHAPE;
    const int es = elem_bytes(cfg->dtype), per16 = 16 / es;
    if ((r->A & 15) || (r->B & 15) || (r->C & 15) || r->lda % per16 || r->ldb % per16 || r->ldc % 8)
        return GEMM_ERR_ALIGN;
    // the kernel addresses a tile's operands with 32-bit byte offsets below 2 GiB
    const int64_t lim = (int64_t)1 << 31;
    const int64_t b_window = cfg->b_layout ? (int64_t)v.block_n * r->ldb * es
                                           : (k_per_split(v, r->K, 1) + (int64_t)v.stages * v.block_k) * r->ldb * es;
    if ((int64_t)v.block_m * r->lda * es >= lim || b_window >= lim || (int64_t)r->tiles_m * r->tiles_n >= lim)
        return GEMM_ERR_SHAPE;
    return GEMM_OK;
}
}  // namespace g355

namespace {
// shapes of the problems, or a gemm_status for the first one that is not a legal group
int group_shapes(int n_groups, const gemm_problem *problems, int dtype, int b_layout, GroupShape *shapes,
                 int64_t *m_max, int64_t *n_max, int64_t *k_max, bool all_empty_ok = false)
{
    if (!problems)
        return GEMM_ERR_NULL;
    if (n_groups < 1 || n_groups > kMaxGroups)
        return GEMM_ERR_SHAPE;
    if (b_layout != GEMM_B_ROW_MAJOR && b_layout != GEMM_B_K_CONTIGUOUS)
        return GEMM_ERR_CFG_ILLEGAL;
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3 && dtype != GEMM_FP16)
        return GEMM_ERR_DTYPE;
    *m_max = *n_max = *k_max = 0;
    for (int i = 0; i < n_groups; ++i) {
        if (problems[i].M < 0)
            return GEMM_ERR_SHAPE;
        // an empty group still names a well-formed N and K
        const int rc = check_problem(problems[i].M > 0 ? problems[i].M : 1, problems[i].N, problems[i].K, dtype);
        if (rc)
            return rc;
        shapes[i].M = problems[i].M;
        shapes[i].N = problems[i].N;
        shapes[i].K = problems[i].K;
        if (problems[i].M > 0) {
            *m_max = problems[i].M > *m_max ? problems[i].M : *m_max;
            *n_max = problems[i].N > *n_max ? problems[i].N : *n_max;
            *k_max = problems[i].K > *k_max ? problems[i].K : *k_max;
        }
    }
    if (*m_max == 0 && !all_empty_ok)
        return GEMM_ERR_SHAPE;   // every group is empty: nothing to select for
    return GEMM_OK;
}

void fill_grouped_cfg(const gemm_hw &hw, int dtype, int b_layout, int id, int n_groups, int64_t m_max, int64_t n_max,
                      int64_t k_max, double l_total, int bottleneck, gemm_cfg *out)
{
    fill_cfg(hw, dtype, b_layout, m_max, n_max, k_max, id, 1, 0, out, 1);
    out->groups = n_groups;
    out->bottleneck = bottleneck;
    out->predicted_us = l_total / (hw.clk_ghz * 1e3);
}
}  // namespace

extern "C" {

int gemm_variant_count(int dtype)
{
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3 && dtype != GEMM_FP16)
        return GEMM_ERR_DTYPE;
    return variant_count(dtype);
}

int gemm_cfg_at_grouped(int variant, int n_groups, const gemm_problem *problems, int dtype, int b_layout, gemm_cfg *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    GroupShape shapes[kMaxGroups];
    int64_t mm, nm, km;
    const int rc = group_shapes(n_groups, problems, dtype, b_layout, shapes, &mm, &nm, &km);
    if (rc)
        return rc;
    if (variant < 0 || variant >= variant_count(dtype))
        return GEMM_ERR_INDEX;
    const gemm_hw &hw = hw_current();
    double l_total;
    int label;
    if (!predict_grouped(hw, dtype, b_layout, n_groups, shapes, variant_at(dtype, variant), &l_total, &label, nullptr))
        return GEMM_ERR_CFG_ILLEGAL;
    fill_grouped_cfg(hw, dtype, b_layout, variant, n_groups, mm, nm, km, l_total, label, out);
    return GEMM_OK;
}

int gemm_select_grouped(int n_groups, const gemm_problem *problems, int dtype, int b_layout, gemm_cfg *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    GroupShape shapes[kMaxGroups];
    int64_t mm, nm, km;
    const int rc = group_shapes(n_groups, problems, dtype, b_layout, shapes, &mm, &nm, &km);
    if (rc)
        return rc;
    const gemm_hw &hw = hw_current();
    int best_id = -1, best_label = 0;
    double best = 0.0;
    // fixed enumeration order and a strict '<': the first of equal predictions wins (on K-contiguous B one
    // listed variant goes before the entry it ties with, see variant_wins_tie_on_kc)
    for (int id = 0; id < variant_count(dtype); ++id) {
        double l_total;
        int label;
        if (!predict_grouped(hw, dtype, b_layout, n_groups, shapes, variant_at(dtype, id), &l_total, &label, nullptr))
            continue;
        if (best_id < 0 || l_total < best) {
            best = l_total;
            best_id = id;
            best_label = label;
        }
    }
    if (best_id < 0)
        return GEMM_ERR_CFG_ILLEGAL;
    fill_grouped_cfg(hw, dtype, b_layout, best_id, n_groups, mm, nm, km, best, best_label, out);
    return GEMM_OK;
}

int gemm_grouped_plan(const gemm_cfg *cfg, int n_groups, const gemm_problem *problems, gemm_group_rec *table_out,
                      int64_t *workgroups_out)
{
    if (!cfg || !problems || !table_out || !workgroups_out)
        return GEMM_ERR_NULL;
    int rc = check_grouped_cfg(cfg, n_groups);
    if (rc)
        return rc;
    GroupShape shapes[kMaxGroups];
    int64_t mm, nm, km;
    rc = group_shapes(n_groups, problems, cfg->dtype, cfg->b_layout, shapes, &mm, &nm, &km, true);
    if (rc)
        return rc;
    const Variant &v = variant_at(cfg->dtype, cfg->kernel_id);
    int group_m[kMaxGroups];
    double l_total;
    int label;
    if (mm == 0) {
        for (int i = 0; i < n_groups; ++i)
            group_m[i] = 1;   // every group is empty: a plan without tiles
    } else if (!predict_grouped(hw_current(), cfg->dtype, cfg->b_layout, n_groups, shapes, v, &l_total, &label, group_m)) {
        return GEMM_ERR_CFG_ILLEGAL;
    }
    // Tiles are dispatched in id order, so the groups with the longest K loops go first and the
    // short tiles of the other groups fill the end of the launch (records carry their own
    // pointers: their order in the table is free).  Stable: equal K keeps the caller's order.
    int order[kMaxGroups];
    for (int i = 0; i < n_groups; ++i)
        order[i] = i;
    std::stable_sort(order, order + n_groups, [&](int a, int b) { return problems[a].K > problems[b].K; });
    const int64_t lim = (int64_t)1 << 31;
    const int X = grouped_xcds(cfg);
    int64_t start = 0;   // per-XCD slots taken so far
    for (int j = 0; j < n_groups; ++j) {
        const int i = order[j];
        const gemm_problem &p = problems[i];
        gemm_group_rec r;
        std::memset(&r, 0, sizeof(r));
        if (p.lda >= lim || p.ldb >= lim || p.ldc >= lim || p.lda < 0 || p.ldb < 0 || p.ldc < 0)
            return GEMM_ERR_SHAPE;
        r.A = (uint64_t)(uintptr_t)p.A;
        r.B = (uint64_t)(uintptr_t)p.B;
        r.C = (uint64_t)(uintptr_t)p.C;
        r.M = (int32_t)p.M;
        r.N = (int32_t)p.N;
        r.K = (int32_t)p.K;
        r.lda = (int32_t)p.lda;
        r.ldb = (int32_t)p.ldb;
        r.ldc = (int32_t)p.ldc;
        r.tiles_m = (int32_t)((p.M + v.block_m - 1) / v.block_m);
        r.tiles_n = (int32_t)((p.N + v.block_n - 1) / v.block_n);
        r.tile_start = (int32_t)start;
        r.group_m = group_m[i];
        rc = check_group_rec(cfg, &r, start);
        if (rc)
            return rc;
        start += ((int64_t)r.tiles_m * r.tiles_n + X - 1) / X;
        if (start * X >= lim)
            return GEMM_ERR_SHAPE;
        table_out[j] = r;
    }
    *workgroups_out = start * X;
    return GEMM_OK;
}

uint32_t gemm_abi_version(void) { return GEMM_ABI_VERSION; }

const char *gemm_strerror(int status)
{
    switch (status) {
    case GEMM_OK: return "ok";
    case GEMM_ERR_NULL: return "null pointer";
    case GEMM_ERR_SHAPE: return "bad shape";
    case GEMM_ERR_DTYPE: return "unknown dtype";
    case GEMM_ERR_CFG_ILLEGAL: return "configuration is not legal for this problem";
    case GEMM_ERR_ALIGN: return "pointer, leading dimension or batch stride not aligned to 16 bytes";
    case GEMM_ERR_WORKSPACE: return "split-K workspace missing or too small";
    case GEMM_ERR_ABI: return "ABI version mismatch";
    case GEMM_ERR_HIP: return "HIP launch failed";
    case GEMM_ERR_INDEX: return "configuration index out of range";
    default: return "unknown status";
    }
}

int gemm_cfg_count(int dtype)
{
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3 && dtype != GEMM_FP16)
        return GEMM_ERR_DTYPE;
    return variant_count(dtype) * kNumSplits;
}

int gemm_cfg_at(int idx, int64_t M, int64_t N, int64_t K, int dtype, gemm_cfg *out)
{
    return gemm_cfg_at_ex(idx, M, N, K, dtype, GEMM_B_ROW_MAJOR, out);
}

int gemm_cfg_at_ex(int idx, int64_t M, int64_t N, int64_t K, int dtype, int b_layout, gemm_cfg *out)
{
    return gemm_cfg_at_batched(idx, M, N, K, 1, dtype, b_layout, out);
}

int gemm_cfg_at_batched(int idx, int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int b_layout, gemm_cfg *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    if (batch < 1 || batch > 65535)
        return GEMM_ERR_SHAPE;
    if (b_layout != GEMM_B_ROW_MAJOR && b_layout != GEMM_B_K_CONTIGUOUS)
        return GEMM_ERR_CFG_ILLEGAL;
    const int rc = check_problem(M, N, K, dtype);
    if (rc)
        return rc;
    if (idx < 0 || idx >= variant_count(dtype) * kNumSplits)
        return GEMM_ERR_INDEX;
    const int id = idx / kNumSplits, split = split_k_of(idx % kNumSplits), sk = stream_k_of(idx % kNumSplits);
    const gemm_hw &hw = hw_current();
    if (!variant_legal(hw, variant_at(dtype, id), dtype, M, N, K, split, sk, batch))
        return GEMM_ERR_CFG_ILLEGAL;
    fill_cfg(hw, dtype, b_layout, M, N, K, id, split, sk, out, batch);
    return GEMM_OK;
}

int gemm_select(int64_t M, int64_t N, int64_t K, int dtype, gemm_cfg *out)
{
    return gemm_select_ex(M, N, K, dtype, GEMM_B_ROW_MAJOR, out);
}

int gemm_select_ex(int64_t M, int64_t N, int64_t K, int dtype, int b_layout, gemm_cfg *out)
{
    return gemm_select_batched(M, N, K, 1, dtype, b_layout, out);
}

int gemm_select_batched(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int b_layout, gemm_cfg *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    if (batch < 1 || batch > 65535)
        return GEMM_ERR_SHAPE;
    if (b_layout != GEMM_B_ROW_MAJOR && b_layout != GEMM_B_K_CONTIGUOUS)
        return GEMM_ERR_CFG_ILLEGAL;
    const int rc = check_problem(M, N, K, dtype);
    if (rc)
        return rc;
    const gemm_hw &hw = hw_current();
    int best_id = -1, best_mode = 0;
    double best = 0.0;
    // fixed enumeration order and a strict '<': the first of equal predictions wins
    for (int id = 0; id < variant_count(dtype); ++id) {
        const Variant &v = variant_at(dtype, id);
        FactorPairs pairs;
        for (int s = 0; s < kNumSplits; ++s) {
            if (!variant_legal(hw, v, dtype, M, N, K, split_k_of(s), stream_k_of(s), batch))
                continue;
            gemm_prediction p;
            int gm, gn;
            predict(hw, dtype, b_layout, M, N, K, v, split_k_of(s), stream_k_of(s), &p, &gm, &gn, batch, nullptr, &pairs);
            const bool tie_kc = best_id >= 0 && b_layout == GEMM_B_K_CONTIGUOUS && dtype != GEMM_FP8_E4M3 &&
                                p.l_total == best && s == best_mode && variant_wins_tie_on_kc(v) &&
                                !variant_wins_tie_on_kc(variant_at(dtype, best_id));
            if (best_id < 0 || p.l_total < best || tie_kc) {
                best = p.l_total;
                best_id = id;
                best_mode = s;
            }
        }
    }
    if (best_id < 0)
        return GEMM_ERR_CFG_ILLEGAL;
    fill_cfg(hw, dtype, b_layout, M, N, K, best_id, split_k_of(best_mode), stream_k_of(best_mode), out, batch);
    return GEMM_OK;
}

int gemm_predict(const gemm_cfg *cfg, gemm_prediction *out)
{
    if (!cfg || !out)
        return GEMM_ERR_NULL;
    if (cfg->abi_version != GEMM_ABI_VERSION)
        return GEMM_ERR_ABI;
    const int rc = check_problem(cfg->M, cfg->N, cfg->K, cfg->dtype);
    if (rc)
        return rc;
    if (cfg->kernel_id < 0 || cfg->kernel_id >= variant_count(cfg->dtype))
        return GEMM_ERR_CFG_ILLEGAL;
    const gemm_hw &hw = hw_current();
    const Variant &v = variant_at(cfg->dtype, cfg->kernel_id);
    if (!variant_legal(hw, v, cfg->dtype, cfg->M, cfg->N, cfg->K, cfg->split_k, cfg->stream_k, cfg->batch))
        return GEMM_ERR_CFG_ILLEGAL;
    int gm, gn;
    if (cfg->b_layout > 1 || cfg->stream_k > 1)
        return GEMM_ERR_CFG_ILLEGAL;
    predict(hw, cfg->dtype, cfg->b_layout, cfg->M, cfg->N, cfg->K, v, cfg->split_k, cfg->stream_k, out, &gm, &gn,
            cfg->batch);
    return GEMM_OK;
}

int gemm_grouped_locate(const gemm_cfg *cfg, int n_groups, const gemm_group_rec *table, int64_t workgroup, int32_t out3[3])
{
    if (!cfg || !table || !out3)
        return GEMM_ERR_NULL;
    int rc = check_grouped_cfg(cfg, n_groups);
    if (rc)
        return rc;
    const int X = grouped_xcds(cfg);
    int64_t slots = 0;
    for (int i = 0; i < n_groups; ++i) {
        rc = check_group_rec(cfg, &table[i], slots);
        if (rc)
            return rc;
        slots += group_slots((int64_t)table[i].tiles_m * table[i].tiles_n, X);
    }
    if (workgroup < 0 || workgroup >= slots * X)
        return GEMM_ERR_INDEX;
    // the kernel's own steps, on the host
    const GroupRec *tab = reinterpret_cast<const GroupRec *>(table);
    const int x = (int)(workgroup % X), q = (int)(workgroup / X);
    const int gi = group_of(tab, n_groups, q);
    const GroupRec &r = tab[gi];
    const int t = group_tile(r.tiles_m * r.tiles_n, X, x, q - r.tile_start);
    out3[0] = t < 0 ? -1 : gi;
    out3[1] = out3[2] = -1;
    if (t >= 0) {
        int tm, tn;
        logical_tile(r.tiles_m, r.tiles_n, r.group_m, t, tm, tn);
        out3[1] = tm;
        out3[2] = tn;
    }
    return GEMM_OK;
}

int gemm_stream_k_contributors(const gemm_cfg *cfg, int sk_tile, int32_t out3[3])
{
    if (!cfg || !out3)
        return GEMM_ERR_NULL;
    if (cfg->abi_version != GEMM_ABI_VERSION)
        return GEMM_ERR_ABI;
    SkPlan p;
    if (!cfg_stream_k_plan(cfg, &p))
        return GEMM_ERR_CFG_ILLEGAL;
    if (sk_tile < 0 || sk_tile >= p.sk_tiles)
        return GEMM_ERR_INDEX;
    int a, b;
    sk_contributors(p, sk_tile, &a, &b);
    out3[0] = a;
    out3[1] = b;
    out3[2] = sk_slot_of(p, a, sk_tile);
    return GEMM_OK;
}

int gemm_hw_get(gemm_hw *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    *out = hw_current();
    return GEMM_OK;
}

int gemm_hw_set(const gemm_hw *in)
{
    if (!in)
        return GEMM_ERR_NULL;
    if (in->n_cu < 1 || in->n_xcd < 1 || in->n_cu % in->n_xcd || in->simd_per_cu < 1 || in->clk_ghz <= 0 ||
        in->hbm_bytes_per_clk <= 0 || in->mall_bytes_per_clk <= 0 || in->l2_bytes_per_clk <= 0 ||
        in->lds_bytes_per_clk <= 0 || in->lds_tr_bytes_per_clk <= 0 || in->vmem_bytes_per_clk <= 0 ||
        in->lds_bytes <= 0 || in->under_occ_frac <= 0 || in->under_occ_frac > 1 || in->seg_eff_lo <= 0 || in->seg_eff_lo > 1 ||
        in->overlap_frac < 0 || in->overlap_frac > 1 || in->fill_issue_bytes_per_clk <= 0 || in->slab_sync_clk < 0 ||
        in->n_cu > 4096 || in->simd_per_cu > 64)
        return GEMM_ERR_SHAPE;
    for (int d = 0; d < 2; ++d)
        for (int m = 0; m < 2; ++m)
            if (!(in->l_mi_clk[d][m] > 0))
                return GEMM_ERR_SHAPE;
    hw_replace(*in);
    return GEMM_OK;
}

int gemm_hw_reset(void)
{
    hw_reset();
    return GEMM_OK;
}

int gemm_hw_preset(int id, gemm_hw *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    return hw_preset(id, out) ? GEMM_OK : GEMM_ERR_INDEX;
}

size_t gemm_workspace_bytes(const gemm_cfg *cfg)
{
    if (!cfg || cfg->M < 1 || cfg->N < 1)
        return 0;
    if (cfg->stream_k)
        return (size_t)2 * cfg->sk_workers * cfg->block_m * cfg->block_n * sizeof(float);
    if (cfg->split_k <= 1)
        return 0;
    // slab rows are N rounded up to 8 floats apart
    return (size_t)(cfg->batch > 1 ? cfg->batch : 1) * cfg->split_k * (size_t)cfg->M * (size_t)((cfg->N + 7) / 8 * 8) * sizeof(float);
}

int gemm_stream_k_plan(const gemm_cfg *cfg, int32_t plan4[4])
{
    if (!cfg || !plan4)
        return GEMM_ERR_NULL;
    if (cfg->abi_version != GEMM_ABI_VERSION)
        return GEMM_ERR_ABI;
    SkPlan p;
    if (!cfg_stream_k_plan(cfg, &p))
        return GEMM_ERR_CFG_ILLEGAL;
    plan4[0] = p.workers;
    plan4[1] = p.sk_tiles;
    plan4[2] = p.dp_tiles;
    plan4[3] = p.slabs;
    return GEMM_OK;
}

int gemm_stream_k_segments(const gemm_cfg *cfg, int worker, gemm_sk_segment seg[2])
{
    if (!cfg || !seg)
        return GEMM_ERR_NULL;
    if (cfg->abi_version != GEMM_ABI_VERSION)
        return GEMM_ERR_ABI;
    SkPlan p;
    if (!cfg_stream_k_plan(cfg, &p))
        return GEMM_ERR_CFG_ILLEGAL;
    if (worker < 0 || worker >= p.workers)
        return GEMM_ERR_INDEX;
    SkSegment s[2];
    const int n = sk_segments(p, worker, s);
    const int tiles_m = (int)((cfg->M + cfg->block_m - 1) / cfg->block_m);
    const int tiles_n = (int)((cfg->N + cfg->block_n - 1) / cfg->block_n);
    for (int i = 0; i < n; ++i) {
        int tm, tn;
        logical_tile(tiles_m, tiles_n, cfg->group_m, p.dp_tiles + s[i].tile, tm, tn);
        seg[i].tile_m = tm;
        seg[i].tile_n = tn;
        seg[i].slab0 = s[i].slab0;
        seg[i].count = s[i].count;
        seg[i].complete = s[i].complete;
        seg[i].sk_tile = s[i].tile;
    }
    return n;
}

}  // extern "C"
