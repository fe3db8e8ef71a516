// Analytical latency model and selector (host only; no HIP call anywhere in this file).
//
// Follows Section IV of the paper: Algorithm 3 (compute latency of a workgroup tile),
// Algorithm 4 (waves and active CUs of the last wave), Algorithms 5/6 (cache-tile
// factorisations and hit rate) with the capacity derate of Section IV-C, Algorithm 7
// (memory latency of one K iteration), Algorithm 8 (output-tile latency) and Algorithm 9
// (total latency).  Quantities are bytes and compute clocks.  Where the paper leaves a step
// open the choice made here is stated next to the code.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "../../include/gemm.h"
#include "model.hpp"
#include "stream_k.hpp"
#include "variants.hpp"

namespace g355 {

#define G355_X(bm, bn, bk, wm, wn, mi, ns, lf, lf_kc) {bm, bn, bk, wm, wn, mi, ns},
static const Variant kVariantsBf16[] = {G355_VARIANTS_BF16(G355_X)};
static const Variant kVariantsFp8[] = {G355_VARIANTS_FP8(G355_X)};
#undef G355_X

int variant_count(int dtype)
{
    // fp16 runs the bf16 tile list (same data path, same matrix-core rate)
    return dtype != GEMM_FP8_E4M3 ? (int)(sizeof(kVariantsBf16) / sizeof(Variant))
                                  : (int)(sizeof(kVariantsFp8) / sizeof(Variant));
}
const Variant &variant_at(int dtype, int id)
{
    return dtype != GEMM_FP8_E4M3 ? kVariantsBf16[id] : kVariantsFp8[id];
}

// One MI355X.  Measured with the library's probes (calibrate.py --rates-only): the matrix-instruction
// issue intervals (register-resident MFMA loop on workload-like operands, in the settled state, expressed
// in 2.4 GHz clocks: the chip is power-limited, so this is what an instruction costs while the datapath
// toggles), the LDS fragment-read rates and the HBM rate.  The remaining rates and fixed costs are
// effective values fitted against sweeps of this kernel family; the probes' raw figures for them
// (L2 1610 B/clk per XCD, MALL 2940, idle load latency 960 clk) are upper bounds that the kernels, with
// their MFMA work going on beside the loads, do not reach.
static gemm_hw make_default_hw()
{
    gemm_hw h;
    std::memset(&h, 0, sizeof(h));
    h.n_cu = 256;
    h.n_xcd = 8;
    h.simd_per_cu = 4;
    h.lds_bytes = 160.0 * 1024;
    h.l2_bytes = 4.0 * 1024 * 1024;
    h.mall_bytes = 256.0 * 1024 * 1024;
    h.clk_ghz = 2.4;
    h.hbm_bytes_per_clk = 2700.0;    // 6.5 TB/s: the streaming-read probe's rate, of the 8 TB/s pins
    h.mall_bytes_per_clk = 2400.0;   // what L2 misses are served at when the MALL holds the data (fitted; a streaming read sees 6.5 TB/s)
    h.l2_bytes_per_clk = 2048.0;     // 16 channels x 128 B per XCD
    h.lds_bytes_per_clk = 250.0;     // ds_read_b128 fragments (probe: 153 TB/s over 256 CUs)
    h.lds_tr_bytes_per_clk = 222.0;  // ds_read_b64_tr_* fragments (probe: 136 TB/s)
    h.vmem_bytes_per_clk = 25.3;     // Algorithm 7's R_L1: fill rate a CU sustains when loads are what it waits for (fitted)
    h.fill_issue_bytes_per_clk = 55.0;  // wave time the fill of a slab takes out of the MFMA stream (fitted; the vector-memory path issues at most 64 B/clk)
    h.slab_sync_clk = 95.0;          // barrier and first-fragment wait per slab (fitted)
    h.mem_latency_clk = 1350.0;
    h.cache_eff_frac = 0.175;
    h.launch_clk = 2600.0;
    h.wg_overhead_clk = 330.0;
    h.epilogue_clk = 425.0;
    h.reduce_launch_clk = 10600.0;   // 4.4 us: the second launch of a split-K or stream-K run
    h.under_occ_frac = 0.85;
    h.seg_eff_lo = 0.105;
    h.overlap_frac = 0.5;            // fitted
    // on N(0,1)-like operands; on constant operands the four reach 2440 / 2440 / 4930 / 4940 TFLOP/s (32.9 / 16.5 / 65.3 / 32.6 clk)
    h.l_mi_clk[GEMM_BF16][0] = 44.4;      // v_mfma_f32_32x32x16_bf16  (1812 TFLOP/s device-wide)
    h.l_mi_clk[GEMM_BF16][1] = 19.6;      // v_mfma_f32_16x16x32_bf16  (2054 TFLOP/s)
    h.l_mi_clk[GEMM_FP8_E4M3][0] = 81.7;  // v_mfma_f32_32x32x64_f8f6f4 (3940 TFLOP/s)
    h.l_mi_clk[GEMM_FP8_E4M3][1] = 37.8;  // v_mfma_f32_16x16x128_f8f6f4 (4264 TFLOP/s)
    return h;
}

// A 304-CU CDNA3-class part as the paper's evaluation platform (Section V): public sizes and
// bandwidths; matrix instructions at half the per-CU rate and half the LDS read width; fixed costs
// left as fitted here.  Nothing in it is a timing of this library's kernels.
static gemm_hw make_mi300x_like_hw()
{
    gemm_hw h = make_default_hw();
    h.n_cu = 304;
    h.n_xcd = 8;
    h.lds_bytes = 64.0 * 1024;
    h.clk_ghz = 2.1;
    h.hbm_bytes_per_clk = 5300.0 * 0.75 / 2.1;   // 5.3 TB/s pins, three quarters sustained
    h.mall_bytes_per_clk = 17200.0 / 2.1 * 0.6;  // 17.2 TB/s peak Infinity Cache rate
    h.lds_bytes_per_clk = 125.0;
    h.lds_tr_bytes_per_clk = 30.0;               // no transpose LDS reads: narrow reads instead
    for (int d = 0; d < 2; ++d)
        for (int m = 0; m < 2; ++m)
            h.l_mi_clk[d][m] = 2.0 * make_default_hw().l_mi_clk[d][m];
    return h;
}

bool hw_preset(int id, gemm_hw *out)
{
    if (id == GEMM_HW_MI355X)
        *out = make_default_hw();
    else if (id == GEMM_HW_MI300X_LIKE)
        *out = make_mi300x_like_hw();
    else
        return false;
    return true;
}

static gemm_hw g_hw = make_default_hw();

const gemm_hw &hw_current() { return g_hw; }
void hw_replace(const gemm_hw &h) { g_hw = h; }
void hw_reset() { g_hw = make_default_hw(); }

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

int elem_bytes(int dtype) { return dtype == GEMM_FP8_E4M3 ? 1 : 2; }

int mfma_k(int dtype, int mfma)
{
    if (dtype != GEMM_FP8_E4M3)
        return mfma == 32 ? 16 : 32;
    return mfma == 32 ? 64 : 128;
}

int64_t k_per_split(const Variant &v, int64_t K, int split_k)
{
    return cdiv(cdiv(K, v.block_k), split_k) * v.block_k;
}

static int occupancy(const gemm_hw &hw, const Variant &v, int dtype);

int stream_k_workers(const gemm_hw &hw, const Variant &v, int dtype) { return hw.n_cu * occupancy(hw, v, dtype); }

bool variant_legal(const gemm_hw &hw, const Variant &v, int dtype, int64_t M, int64_t N, int64_t K, int split_k,
                   int stream_k, int64_t batch)
{
    const int es = elem_bytes(dtype);
    if (batch < 1 || batch > 65535 || (stream_k && batch != 1))
        return false;
    if (stream_k) {
        // stream-K splits the last partial wave of tiles; it needs one, and work for every worker
        SkPlan plan;
        if (split_k != 1 || !sk_make_plan(cdiv(M, v.block_m) * cdiv(N, v.block_n), stream_k_workers(hw, v, dtype),
                                          cdiv(K, v.block_k), &plan))
            return false;
    }
    const double lds = (double)v.stages * (v.block_m + v.block_n) * v.block_k * es;
    if (lds > hw.lds_bytes)
        return false;
    if (split_k < 1)
        return false;
    if (split_k > 1) {
        // every K slice must own at least one slab
        const int64_t kps = k_per_split(v, K, split_k);
        if ((int64_t)(split_k - 1) * kps >= K)
            return false;
    }
    return true;
}

// Workgroups of this variant that fit one CU at a time (LDS, registers, wave slots).
static int occupancy(const gemm_hw &hw, const Variant &v, int dtype)
{
    const int es = elem_bytes(dtype);
    const double lds = (double)v.stages * (v.block_m + v.block_n) * v.block_k * es;
    const int waves = v.waves_m * v.waves_n;
    const int nt = waves * 64;
    // registers per lane: fp32 accumulators + staged slab + fragments and addresses
    const double acc = (double)v.block_m * v.block_n / nt;
    const double vgpr = acc + 64.0;
    int waves_per_simd = (int)std::floor(512.0 / vgpr);
    waves_per_simd = std::max(1, std::min(8, waves_per_simd));
    const int by_regs = std::max(1, waves_per_simd * hw.simd_per_cu / waves);
    const int by_lds = std::max(1, (int)std::floor(hw.lds_bytes / lds));
    return std::max(1, std::min(std::min(by_regs, by_lds), 8));
}

// Algorithm 5 with the cache tile clipped to the tile grid.
static double hit_rate(double f_m, double f_n, double bm, double bn)
{
    const double u = f_m * bm + f_n * bn;
    const double r = f_m * f_n * (bm + bn);
    if (r <= 0)
        return 0.0;
    const double h = 1.0 - u / r;
    return std::min(1.0, std::max(0.0, h));
}

// Algorithm 6 + the choice of the pair: among all (f_m, f_n) with f_m * f_n = scope, clipped
// to the tile grid, take the one with the highest Algorithm-5 hit rate; ties go to the pair
// whose cache tile is closest to square in elements, then to the wider one.
static void best_factor_pair(int scope, const Variant &v, int64_t tiles_m, int64_t tiles_n, double *fm_out,
                             double *fn_out, int *fm_raw_out)
{
    double best_h = -1.0, best_fm = 1, best_fn = 1, best_skew = 0;
    int best_raw = 1;
    // all divisors i of scope in ascending order (trial division up to sqrt, both cofactors kept)
    int divs[128];
    int nd = 0, nhi = 0;
    int hi[64];
    for (int i = 1; (int64_t)i * i <= scope; ++i) {
        if (scope % i)
            continue;
        divs[nd++] = i;
        if (i != scope / i)
            hi[nhi++] = scope / i;
    }
    while (nhi > 0)
        divs[nd++] = hi[--nhi];
    for (int d = 0; d < nd; ++d) {
        const int i = divs[d];
        const int j = scope / i;
        const double fm = (double)std::min<int64_t>(i, tiles_m);
        const double fn = (double)std::min<int64_t>(j, tiles_n);
        const double h = hit_rate(fm, fn, v.block_m, v.block_n);
        const double skew = std::fabs(fm * v.block_m - fn * v.block_n);
        bool better = false;
        if (h > best_h + 1e-12)
            better = true;
        else if (std::fabs(h - best_h) <= 1e-12) {
            if (skew < best_skew - 1e-9)
                better = true;
            else if (std::fabs(skew - best_skew) <= 1e-9 && fn > best_fn)
                better = true;
        }
        if (better) {
            best_h = h;
            best_fm = fm;
            best_fn = fn;
            best_skew = skew;
            best_raw = i;
        }
    }
    *fm_out = best_fm;
    *fn_out = best_fn;
    *fm_raw_out = best_raw;
}

struct MemTerms {
    double l_issue, l_lds, l_l2, l_mall, l_hbm, l_mem;
};

// Fraction of the HBM rate reached when a tile touches `seg` contiguous bytes of each matrix
// row: 1 from 256 bytes up, falling linearly in log2(seg) to seg_eff_lo at 32 bytes.
static double segment_efficiency(const gemm_hw &hw, double seg)
{
    if (seg >= 256.0)
        return 1.0;
    const double s = std::max(seg, 32.0);
    return std::min(1.0, hw.seg_eff_lo + (1.0 - hw.seg_eff_lo) * std::log2(s / 32.0) / 3.0);
}

// Algorithm 7 for one K iteration.  `per_cu` = tiles a CU works on at once, `active` = CUs
// busy.  Terms: per-CU vector-memory issue, LDS fragment reads (the software-managed-memory
// bound of Section IV-D, which the printed algorithm leaves out), L2 (per XCD), MALL and HBM.
// `bm_e` x `bn_e`: mean valid extent of a tile (rows and columns outside the matrix are never
// fetched); `per_cu_mem`: tiles per CU whose bytes move (fractional in the last wave).
static MemTerms memory_latency(const gemm_hw &hw, const Variant &v, int es, int b_layout, double per_cu, double active,
                               double h1, double h2, double bm_e, double bn_e, double per_cu_mem, double ea, double eb)
{
    MemTerms t;
    // every load instruction of the nominal tile is issued; only the valid extent moves bytes
    t.l_issue = (double)(v.block_m + v.block_n) * v.block_k * es * per_cu / hw.vmem_bytes_per_clk;
    const double a_bytes = bm_e * v.block_k * es * per_cu_mem;   // per CU and iteration
    const double b_bytes = bn_e * v.block_k * es * per_cu_mem;
    const double ld_cu = a_bytes + b_bytes;
    // every wave reads its A rows (ds_read_b128) and its B columns (transpose reads, or
    // ds_read_b128 when B is K-contiguous) of the slab
    const double b_lds_rate = b_layout ? hw.lds_bytes_per_clk : hw.lds_tr_bytes_per_clk;
    t.l_lds = ((double)v.block_m * v.waves_n * v.block_k * es / hw.lds_bytes_per_clk +
               (double)v.block_n * v.waves_m * v.block_k * es / b_lds_rate) *
              per_cu;
    const double xcds_busy = std::min<double>(hw.n_xcd, std::max(1.0, active));   // round-robin dispatch
    const double total = ld_cu * active;
    t.l_l2 = (total / xcds_busy) / hw.l2_bytes_per_clk;
    t.l_mall = (1.0 - h1) * total / hw.mall_bytes_per_clk;
    // what misses both caches, inflated by the row-segment efficiency of each operand
    // (ea, eb: row-segment efficiency of A and B, constant for the variant and layout)
    // Both hit rates come from Algorithm 5 on nested scopes, so h2 already contains the reuse h1
    // counts: the share of requested bytes that reaches HBM is what neither scope can serve,
    // min(1 - h1, 1 - h2), not the product (which could fall below the bytes the matrices hold).
    const double tm = std::min(1.0 - h2, 1.0 - h1) * (a_bytes / ea + b_bytes / eb) * active;
    t.l_hbm = tm / hw.hbm_bytes_per_clk + hw.mem_latency_clk / std::max(1.0, per_cu * (v.stages - 1));
    t.l_mem = std::max(std::max(t.l_issue, t.l_lds), std::max(std::max(t.l_l2, t.l_mall), t.l_hbm));
    return t;
}

static int label_of(const MemTerms &t, double l_comp, bool under, double fixed, double loop)
{
    if (fixed > loop)
        return GEMM_BOUND_LAUNCH;
    if (l_comp >= t.l_mem)
        return under ? GEMM_BOUND_COMPUTE_UNDER : GEMM_BOUND_COMPUTE_FULL;
    if (t.l_mem == t.l_hbm)
        return GEMM_BOUND_HBM;
    if (t.l_mem == t.l_mall)
        return GEMM_BOUND_MALL;
    if (t.l_mem == t.l_l2)
        return GEMM_BOUND_L2;
    if (t.l_mem == t.l_lds)
        return GEMM_BOUND_LDS;
    return GEMM_BOUND_LS_ISSUE;
}

void predict(const gemm_hw &hw, int dtype, int b_layout, int64_t M, int64_t N, int64_t K, const Variant &v, int split_k,
             int stream_k, gemm_prediction *p, int *group_m, int *group_n, int64_t batch, double *l_tile_full_out,
             FactorPairs *pairs)
{
    std::memset(p, 0, sizeof(*p));
    const int es = elem_bytes(dtype);
    const int waves_wg = v.waves_m * v.waves_n;
    const int mi_k = mfma_k(dtype, v.mfma);

    // Algorithm 3: L_MT = N_MI * L_MI, spread over the SIMDs the workgroup's waves occupy.
    const double n_mi = (double)cdiv(v.block_m, v.mfma) * cdiv(v.block_n, v.mfma) * cdiv(v.block_k, mi_k);
    // the fp16 and bf16 matrix instructions issue at the same rate: one row of the table
    const double l_mi = hw.l_mi_clk[dtype == GEMM_FP8_E4M3 ? 1 : 0][v.mfma == 32 ? 0 : 1];
    p->n_mi = n_mi;
    p->l_mt_ideal = n_mi * l_mi / std::min<double>(hw.simd_per_cu, waves_wg);

    // Algorithm 4, with K slices counted as tiles and `occ` workgroups per CU as slots.
    const int64_t tiles_m = cdiv(M, v.block_m), tiles_n = cdiv(N, v.block_n);
    // a batch is that many times the tiles, dispatched back to back in one launch
    const double tiles = (double)tiles_m * tiles_n * split_k * (double)batch;
    const int occ = occupancy(hw, v, dtype);
    const double slots = (double)hw.n_cu * occ;
    const double waves = std::ceil(tiles / slots);
    const double tail_tiles = tiles - (waves - 1) * slots;            // in (0, slots]
    const double active = std::min<double>(tail_tiles, hw.n_cu);      // T_out % N_CU, with 0 read as N_CU
    const double tail_per_cu = std::ceil(tail_tiles / hw.n_cu);
    p->tiles = tiles;
    p->waves = waves;
    p->active_cu = active;
    p->occupancy = occ;

    // Algorithms 5/6: L2 scope = CUs of one XCD (times resident workgroups), MALL scope = device.
    const int l2_scope = hw.n_cu / hw.n_xcd * occ;
    double fm, fn, fm2, fn2;
    int fm_raw, fm2_raw;
    // the pairs depend on the variant and the tile grid only: the K splits of one variant share them
    if (pairs && pairs->valid) {
        fm = pairs->fm[0], fn = pairs->fn[0], fm_raw = pairs->raw[0];
        fm2 = pairs->fm[1], fn2 = pairs->fn[1], fm2_raw = pairs->raw[1];
    } else {
        best_factor_pair(l2_scope, v, tiles_m, tiles_n, &fm, &fn, &fm_raw);
        best_factor_pair(hw.n_cu * occ, v, tiles_m, tiles_n, &fm2, &fn2, &fm2_raw);
        if (pairs) {
            pairs->fm[0] = fm, pairs->fn[0] = fn, pairs->raw[0] = fm_raw;
            pairs->fm[1] = fm2, pairs->fn[1] = fn2, pairs->raw[1] = fm2_raw;
            pairs->valid = true;
        }
    }
    // unique / requested counts of Algorithm 5 on the mean valid extent of a tile
    const double bm_e = (double)M / tiles_m, bn_e = (double)N / tiles_n;
    double h1 = hit_rate(fm, fn, bm_e, bn_e);
    double h2 = hit_rate(fm2, fn2, bm_e, bn_e);
    // Capacity derate: the working set of one K step of the cache tile (two slabs in flight)
    // against the usable share of the cache; beyond it the hit rate shrinks in proportion.
    const double fp1 = (fm * v.block_m + fn * v.block_n) * v.block_k * es * 2.0;
    const double fp2 = (fm2 * v.block_m + fn2 * v.block_n) * v.block_k * es * 2.0;
    h1 *= std::min(1.0, hw.cache_eff_frac * hw.l2_bytes / fp1);
    h2 *= std::min(1.0, hw.cache_eff_frac * hw.mall_bytes / fp2);
    p->f_m = fm;
    p->f_n = fn;
    p->h_l2 = h1;
    p->h_mall = h2;
    *group_m = (int)std::max<int64_t>(1, std::min<int64_t>(fm_raw, tiles_m));
    *group_n = std::max(1, l2_scope / fm_raw);

    // K slabs per tile (Algorithm 8's I + 1), with the reduction split over split_k slices.
    const double slabs = (double)(k_per_split(v, K, split_k) / v.block_k);
    p->iters = slabs - 1.0;
    const double out_bytes = (split_k > 1) ? 4.0 : 2.0;

    const double fill_bytes = (double)(v.block_m + v.block_n) * v.block_k * es;   // one slab of one tile
    // (K-contiguous B under a one-row grid: each piece of a row is read once, by one workgroup, whose next slab
    // continues the row where this one ended -- twice the piece counts)
    const double ea = segment_efficiency(hw, (double)v.block_k * es);
    const double eb = segment_efficiency(hw, (double)(b_layout ? (tiles_m == 1 ? 2 : 1) * v.block_k : v.block_n) * es);
    auto tile_latency = [&](double per_cu, double act, double per_cu_mem, MemTerms *mt_out, double *l_comp_out,
                            double *pro, double *epi, double *iter) {
        // Compute latency of one K slab of one tile: Algorithm 3's L_MT, plus what the slab's fill and
        // its barrier take out of the waves' instruction streams (the direct-to-LDS loads of a slab are
        // issued by the same waves, in order with their MFMAs, and the vector-memory path accepts them at
        // fill_issue_bytes_per_clk; measured slab costs of all variants follow L_MT + fill + a constant).
        // per_cu tiles share the CU; fewer than fit run a little faster each, but not in proportion.
        double l_comp = (p->l_mt_ideal + fill_bytes / hw.fill_issue_bytes_per_clk + hw.slab_sync_clk) * per_cu;
        if (per_cu < occ)
            l_comp *= hw.under_occ_frac + (1.0 - hw.under_occ_frac) * per_cu / occ;
        const MemTerms mt = memory_latency(hw, v, es, b_layout, per_cu, act, h1, h2, bm_e, bn_e, per_cu_mem, ea, eb);
        const double l_pro = mt.l_mem + hw.mem_latency_clk + hw.wg_overhead_clk;
        // the store stage scales with the output tile only; results leave through HBM
        const double l_epi = act * per_cu * v.block_m * v.block_n * out_bytes / hw.hbm_bytes_per_clk + hw.epilogue_clk;
        const double l_iter = std::max(l_comp, mt.l_mem);
        *mt_out = mt;
        *l_comp_out = l_comp;
        *pro = l_pro;
        *epi = l_epi;
        *iter = l_iter;
        // I iterations overlap load and compute; the last slab's compute is exposed
        return l_pro + l_epi + l_iter * (slabs - 1.0) + l_comp;
    };

    MemTerms mt_full, mt_tail;
    double lc_full, lc_tail, pro, epi, iter, pro_t, epi_t, iter_t;
    const double l_tile_full = tile_latency((double)occ, (double)hw.n_cu, (double)occ, &mt_full, &lc_full, &pro, &epi, &iter);
    // the last wave moves the bytes of the tiles that exist: tail / active per CU
    const double l_tile_tail =
        tile_latency(tail_per_cu, active, tail_tiles / active, &mt_tail, &lc_tail, &pro_t, &epi_t, &iter_t);
    if (l_tile_full_out)
        *l_tile_full_out = l_tile_full;
    const bool has_full = waves > 1.0;
    const MemTerms &mt = has_full ? mt_full : mt_tail;
    p->l_compute = has_full ? lc_full : lc_tail;
    p->l_issue = mt.l_issue;
    p->l_lds = mt.l_lds;
    p->l_l2 = mt.l_l2;
    p->l_mall = mt.l_mall;
    p->l_hbm = mt.l_hbm;
    p->l_mem = mt.l_mem;
    p->l_mem_tail = mt_tail.l_mem;
    p->l_prologue = has_full ? pro : pro_t;
    p->l_epilogue = has_full ? epi : epi_t;
    p->l_iter = has_full ? iter : iter_t;
    p->l_tile = has_full ? l_tile_full : l_tile_tail;
    p->l_tile_tail = l_tile_tail;

    // Split-K: a second pass sums the fp32 slabs (read split_k * M * N * 4, write M * N * 2).
    double l_reduce = 0.0;
    if (split_k > 1) {
        const double bytes = (double)M * N * (4.0 * split_k + 2.0) * (double)batch;
        const double rate = (bytes <= hw.cache_eff_frac * hw.mall_bytes) ? hw.mall_bytes_per_clk : hw.hbm_bytes_per_clk;
        l_reduce = hw.reduce_launch_clk + bytes / rate;
    }
    p->l_reduce = l_reduce;

    // Algorithm 9, with full waves and the under-occupied last wave priced separately.  With two or
    // more workgroups resident on a CU, part of a tile's prologue and store stage hides under the K
    // loops of the others whenever another wave of tiles follows.
    const double hidden = (occ >= 2 && has_full) ? hw.overlap_frac * (pro + epi) : 0.0;
    p->l_total = hw.launch_clk + (waves - 1.0) * (l_tile_full - hidden) + l_tile_tail + l_reduce;

    if (stream_k) {
        // Fractional last wave: the tiles % slots tiles left over after the whole waves are cut
        // along K into one equal range of w slabs per slot, so the last "wave" costs w slabs
        // instead of a whole tile.  Every CU is full; a share sk/slots of the workers straddles
        // two tiles and pays the prologue and store stage twice; partial tiles leave as fp32 and a
        // second pass sums them (read (slots + sk) partial tiles, write sk tiles).
        const double sk = std::fmod(tiles, slots);
        const double whole = (tiles - sk) / slots;
        const double w = sk * slabs / slots;
        const double tile_elems = (double)v.block_m * v.block_n;
        // workers that share an L2 are at different K offsets of different tiles: no L2 reuse
        const MemTerms mt_sk =
            memory_latency(hw, v, es, b_layout, (double)occ, (double)hw.n_cu, 0.0, h2, bm_e, bn_e, (double)occ, ea, eb);
        const double iter_sk = std::max(lc_full, mt_sk.l_mem);
        const double pro_sk = mt_sk.l_mem + hw.mem_latency_clk + hw.wg_overhead_clk;
        const double l_epi_sk = hw.n_cu * occ * tile_elems * 4.0 / hw.hbm_bytes_per_clk + hw.epilogue_clk;
        const double l_sk = (1.0 + sk / slots) * (pro_sk + l_epi_sk) + iter_sk * (w - 1.0) + lc_full;
        // second pass: bytes through MALL or HBM, plus the dependent chain of one output's
        // contributors (1, 4 or 8 thread rows share them, 4 loads in flight each)
        const double bytes = (slots + sk) * tile_elems * 4.0 + sk * tile_elems * 2.0;
        const double rate = (bytes <= hw.cache_eff_frac * hw.mall_bytes) ? hw.mall_bytes_per_clk : hw.hbm_bytes_per_clk;
        const double contrib = std::floor(slots / sk) + 2.0;
        const double rows = contrib > 32.0 ? 8.0 : contrib > 8.0 ? 4.0 : 1.0;
        const double chain = std::ceil(contrib / (4.0 * rows)) * hw.mem_latency_clk;
        l_reduce = hw.reduce_launch_clk + bytes / rate + chain;
        p->waves = whole + sk / slots;
        p->active_cu = hw.n_cu;
        p->l_compute = lc_full;
        p->l_issue = mt_full.l_issue;
        p->l_lds = mt_full.l_lds;
        p->l_l2 = mt_full.l_l2;
        p->l_mall = mt_full.l_mall;
        p->l_hbm = mt_full.l_hbm;
        p->l_mem = mt_full.l_mem;
        p->l_mem_tail = mt_full.l_mem;
        p->l_prologue = pro;
        p->l_epilogue = epi;
        p->l_iter = iter;
        p->l_tile = l_tile_full;
        p->l_tile_tail = l_sk;
        p->l_reduce = l_reduce;
        p->l_total = hw.launch_clk + whole * l_tile_full + l_sk + l_reduce;
    }
    p->total_us = p->l_total / (hw.clk_ghz * 1e3);
    const double fixed = hw.launch_clk + l_reduce + waves * (p->l_prologue + p->l_epilogue);
    p->bottleneck = label_of(stream_k ? mt_full : mt, p->l_compute, !stream_k && active < hw.n_cu && waves == 1.0, fixed,
                             p->l_total - fixed);
}

// Grouped launch.  Algorithm 4 on the tiles of all groups together (the launch is one grid);
// Algorithm 8 per group on a full device (other groups' tiles fill the CUs a small group leaves
// free); Algorithm 9 as waves times the tile-weighted mean of the groups' tile latencies.
bool predict_grouped(const gemm_hw &hw, int dtype, int b_layout, int n, const GroupShape *g, const Variant &v,
                     double *l_total_out, int *bottleneck_out, int *group_m_out)
{
    double tiles = 0.0, weighted = 0.0, heaviest = -1.0;
    int label = GEMM_BOUND_LAUNCH;
    for (int i = 0; i < n; ++i) {
        if (group_m_out)
            group_m_out[i] = 1;
        if (g[i].M == 0)
            continue;
        if (!variant_legal(hw, v, dtype, g[i].M, g[i].N, g[i].K, 1, 0, 1))
            return false;
        gemm_prediction p;
        int gm, gn;
        double l_tile = 0.0;
        predict(hw, dtype, b_layout, g[i].M, g[i].N, g[i].K, v, 1, 0, &p, &gm, &gn, 1, &l_tile);
        const double t = (double)cdiv(g[i].M, v.block_m) * (double)cdiv(g[i].N, v.block_n);
        tiles += t;
        weighted += t * l_tile;
        if (t * l_tile > heaviest) {
            heaviest = t * l_tile;
            label = p.bottleneck;
        }
        if (group_m_out)
            group_m_out[i] = gm;
    }
    if (tiles <= 0.0)
        return false;
    const double slots = (double)hw.n_cu * occupancy(hw, v, dtype);
    *l_total_out = hw.launch_clk + std::ceil(tiles / slots) * weighted / tiles;
    if (bottleneck_out)
        *bottleneck_out = label;
    return true;
}

void fill_cfg(const gemm_hw &hw, int dtype, int b_layout, int64_t M, int64_t N, int64_t K, int kernel_id, int split_k,
              int stream_k, gemm_cfg *c, int64_t batch)
{
    const Variant &v = variant_at(dtype, kernel_id);
    gemm_prediction p;
    int gm, gn;
    predict(hw, dtype, b_layout, M, N, K, v, split_k, stream_k, &p, &gm, &gn, batch);
    std::memset(c, 0, sizeof(*c));
    c->abi_version = GEMM_ABI_VERSION;
    c->dtype = dtype;
    c->M = M;
    c->N = N;
    c->K = K;
    // the smallest legal leading dimensions: rows start on 16-byte boundaries (C: 8 elements)
    const int64_t per16 = 16 / elem_bytes(dtype);
    c->lda = cdiv(K, per16) * per16;
    c->ldb = cdiv(b_layout ? K : N, per16) * per16;
    c->ldc = cdiv(N, 8) * 8;
    c->kernel_id = kernel_id;
    c->block_m = (uint16_t)v.block_m;
    c->block_n = (uint16_t)v.block_n;
    c->block_k = (uint16_t)v.block_k;
    c->waves_m = (uint8_t)v.waves_m;
    c->waves_n = (uint8_t)v.waves_n;
    c->mfma = (uint8_t)v.mfma;
    c->k_unroll = (uint8_t)(v.block_k / mfma_k(dtype, v.mfma));
    c->split_k = (uint16_t)split_k;
    c->group_m = (uint16_t)gm;
    c->group_n = (uint16_t)gn;
    c->xcd_remap = 1;
    c->stages = (uint8_t)v.stages;
    c->b_layout = (uint8_t)b_layout;
    c->stream_k = (uint8_t)(stream_k ? 1 : 0);
    c->sk_workers = (uint16_t)(stream_k ? stream_k_workers(hw, v, dtype) : 0);
    c->alpha = 1.0f;
    c->batch = (int32_t)batch;
    c->stride_a = M * c->lda;
    c->stride_b = b_layout ? N * c->ldb : K * c->ldb;
    c->stride_c = M * c->ldc;
    c->bottleneck = p.bottleneck;
    c->predicted_us = p.total_us;
}

}  // namespace g355
