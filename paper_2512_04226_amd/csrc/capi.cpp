// Host-only entry points of the C ABI: selection, enumeration, prediction, hardware
// descriptor.  Nothing here touches the GPU.
#include <cstring>

#include "../../include/gemm.h"
#include "model.hpp"
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
    const int per16 = 16 / elem_bytes(dtype);   // elements per 16-byte chunk
    if (N % per16 || K % per16)
        return GEMM_ERR_ALIGN;
    return GEMM_OK;
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
}  // namespace g355

extern "C" {

uint32_t gemm_abi_version(void) { return GEMM_ABI_VERSION; }

const char *gemm_strerror(int status)
{
    switch (status) {
    case GEMM_OK: return "ok";
    case GEMM_ERR_NULL: return "null pointer";
    case GEMM_ERR_SHAPE: return "bad shape";
    case GEMM_ERR_DTYPE: return "unknown dtype";
    case GEMM_ERR_CFG_ILLEGAL: return "configuration is not legal for this problem";
    case GEMM_ERR_ALIGN: return "pointer, leading dimension, N or K not aligned to 16 bytes";
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
        for (int s = 0; s < kNumSplits; ++s) {
            if (!variant_legal(hw, v, dtype, M, N, K, split_k_of(s), stream_k_of(s), batch))
                continue;
            gemm_prediction p;
            int gm, gn;
            predict(hw, dtype, b_layout, M, N, K, v, split_k_of(s), stream_k_of(s), &p, &gm, &gn, batch);
            if (best_id < 0 || p.l_total < best) {
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
        in->lds_bytes <= 0 || in->under_occ_frac <= 0 || in->under_occ_frac > 1 || in->seg_eff_lo <= 0 || in->seg_eff_lo > 1)
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
    return (size_t)(cfg->batch > 1 ? cfg->batch : 1) * cfg->split_k * (size_t)cfg->M * (size_t)cfg->N * sizeof(float);
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
