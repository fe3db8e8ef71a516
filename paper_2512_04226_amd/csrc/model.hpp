#pragma once
#include <stdint.h>

#include "../../include/gemm.h"
#include "variants.hpp"

namespace g355 {
int variant_count(int dtype);
const Variant &variant_at(int dtype, int id);
const gemm_hw &hw_current();
void hw_replace(const gemm_hw &h);
void hw_reset();
bool hw_preset(int id, gemm_hw *out);
int elem_bytes(int dtype);
int mfma_k(int dtype, int mfma);
int64_t k_per_split(const Variant &v, int64_t K, int split_k);
// stream_k != 0 (with split_k == 1): the last partial wave of tiles is split along K over
// stream_k_workers() workgroups
// batch > 1: that many independent problems of one shape in one launch (no stream-K then)
bool variant_legal(const gemm_hw &hw, const Variant &v, int dtype, int64_t M, int64_t N, int64_t K, int split_k,
                   int stream_k, int64_t batch = 1);
int stream_k_workers(const gemm_hw &hw, const Variant &v, int dtype);
// Algorithm 6's chosen pairs for the L2 and the device scope of one (variant, M, N): a caller that
// evaluates several K splits of one variant passes the same object to reuse them.
struct FactorPairs {
    double fm[2], fn[2];
    int raw[2];
    bool valid = false;
};
void predict(const gemm_hw &hw, int dtype, int b_layout, int64_t M, int64_t N, int64_t K, const Variant &v, int split_k,
             int stream_k, gemm_prediction *p, int *group_m, int *group_n, int64_t batch = 1,
             double *l_tile_full_out = nullptr, FactorPairs *pairs = nullptr);
// Grouped launch of n shapes (M == 0: empty group) with one variant: total latency in clocks, the
// label of the group that weighs most, and each group's rasterisation band height.  False when
// the variant cannot run some group or every group is empty.
struct GroupShape {
    int64_t M, N, K;
};
bool predict_grouped(const gemm_hw &hw, int dtype, int b_layout, int n, const GroupShape *g, const Variant &v,
                     double *l_total_out, int *bottleneck_out, int *group_m_out);
void fill_cfg(const gemm_hw &hw, int dtype, int b_layout, int64_t M, int64_t N, int64_t K, int kernel_id, int split_k,
              int stream_k, gemm_cfg *c, int64_t batch = 1);
// 0 or a gemm_status for the shape / dtype / alignment rules shared by select, cfg_at and run
int check_problem(int64_t M, int64_t N, int64_t K, int dtype);
struct SkPlan;
bool cfg_stream_k_plan(const gemm_cfg *cfg, SkPlan *p);
// 0 or a gemm_status: is `cfg` a grouped cfg for n groups, and does the record (with the tile
// range starting at tile_start) describe a problem its kernel can run?
int check_grouped_cfg(const gemm_cfg *cfg, int n_groups);
int check_group_rec(const gemm_cfg *cfg, const gemm_group_rec *r, int64_t slot_start);
int grouped_xcds(const gemm_cfg *cfg);   // XCDs the groups' tiles are dealt over (1 without the renumbering)
constexpr int kMaxGroups = 4096;
}  // namespace g355
