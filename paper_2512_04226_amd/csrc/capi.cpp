// Host-only entry points of the C ABI: selection, enumeration, prediction, hardware
// descriptor.  Nothing here touches the GPU.
#include <cstring>

#include "../../include/gemm.h"
#include "model.hpp"

using namespace g355;

namespace g355 {
int check_problem(int64_t M, int64_t N, int64_t K, int dtype)
{
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3)
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
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3)
        return GEMM_ERR_DTYPE;
    return variant_count(dtype) * kNumSplitKs;
}

int gemm_cfg_at(int idx, int64_t M, int64_t N, int64_t K, int dtype, gemm_cfg *out)
{
    return gemm_cfg_at_ex(idx, M, N, K, dtype, GEMM_B_ROW_MAJOR, out);
}

int gemm_cfg_at_ex(int idx, int64_t M, int64_t N, int64_t K, int dtype, int b_layout, gemm_cfg *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    if (b_layout != GEMM_B_ROW_MAJOR && b_layout != GEMM_B_K_CONTIGUOUS)
        return GEMM_ERR_CFG_ILLEGAL;
    const int rc = check_problem(M, N, K, dtype);
    if (rc)
        return rc;
    if (idx < 0 || idx >= variant_count(dtype) * kNumSplitKs)
        return GEMM_ERR_INDEX;
    const int id = idx / kNumSplitKs, split = kSplitKs[idx % kNumSplitKs];
    const gemm_hw &hw = hw_current();
    if (!variant_legal(hw, variant_at(dtype, id), dtype, M, N, K, split))
        return GEMM_ERR_CFG_ILLEGAL;
    fill_cfg(hw, dtype, b_layout, M, N, K, id, split, out);
    return GEMM_OK;
}

int gemm_select(int64_t M, int64_t N, int64_t K, int dtype, gemm_cfg *out)
{
    return gemm_select_ex(M, N, K, dtype, GEMM_B_ROW_MAJOR, out);
}

int gemm_select_ex(int64_t M, int64_t N, int64_t K, int dtype, int b_layout, gemm_cfg *out)
{
    if (!out)
        return GEMM_ERR_NULL;
    if (b_layout != GEMM_B_ROW_MAJOR && b_layout != GEMM_B_K_CONTIGUOUS)
        return GEMM_ERR_CFG_ILLEGAL;
    const int rc = check_problem(M, N, K, dtype);
    if (rc)
        return rc;
    const gemm_hw &hw = hw_current();
    int best_id = -1, best_split = 1;
    double best = 0.0;
    // fixed enumeration order and a strict '<': the first of equal predictions wins
    for (int id = 0; id < variant_count(dtype); ++id) {
        const Variant &v = variant_at(dtype, id);
        for (int s = 0; s < kNumSplitKs; ++s) {
            if (!variant_legal(hw, v, dtype, M, N, K, kSplitKs[s]))
                continue;
            gemm_prediction p;
            int gm, gn;
            predict(hw, dtype, b_layout, M, N, K, v, kSplitKs[s], &p, &gm, &gn);
            if (best_id < 0 || p.l_total < best) {
                best = p.l_total;
                best_id = id;
                best_split = kSplitKs[s];
            }
        }
    }
    if (best_id < 0)
        return GEMM_ERR_CFG_ILLEGAL;
    fill_cfg(hw, dtype, b_layout, M, N, K, best_id, best_split, out);
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
    if (!variant_legal(hw, v, cfg->dtype, cfg->M, cfg->N, cfg->K, cfg->split_k))
        return GEMM_ERR_CFG_ILLEGAL;
    int gm, gn;
    if (cfg->b_layout > 1)
        return GEMM_ERR_CFG_ILLEGAL;
    predict(hw, cfg->dtype, cfg->b_layout, cfg->M, cfg->N, cfg->K, v, cfg->split_k, out, &gm, &gn);
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
    if (!cfg || cfg->split_k <= 1 || cfg->M < 1 || cfg->N < 1)
        return 0;
    return (size_t)cfg->split_k * (size_t)cfg->M * (size_t)cfg->N * sizeof(float);
}

}  // extern "C"
