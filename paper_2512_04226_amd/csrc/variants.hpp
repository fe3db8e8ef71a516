// The compiled kernel variants: the candidate tile list the selector ranks (Section V-B of
// the paper speaks of 75 searched configurations; Section V-E of 50-150 valid tiles per
// datatype).  One line per instantiation of gemm_kernel<>:
//   X(BLOCK_M, BLOCK_N, BLOCK_K, WAVES_M, WAVES_N, MFMA, LDS_STAGES, SLAB_CLK, SLAB_CLK_KC)
// SLAB_CLK (B row-major) and SLAB_CLK_KC (B K-contiguous; floored at 0.9 x SLAB_CLK, because the
// larger steady-state gains of the small tiles do not carry over to the small problems that
// use them) are calibration constants of the kernel, measured once on the device like the
// matrix-instruction latency L_MI: 2.4 GHz clocks a CU needs per K_T slab of one workgroup tile
// in steady state (all CUs busy, as many workgroups resident as fit), from an 8192^3 run.
// The order is part of the ABI of kernel_id and of the selector's tie-break (earlier wins).
#pragma once

// bf16: BLOCK_K in elements; MFMA 32 -> v_mfma_f32_32x32x16_bf16, 16 -> v_mfma_f32_16x16x32_bf16
#define G355_VARIANTS_BF16_0(X)    \
    X(256, 256, 64, 2, 4, 32, 2, 4796, 4359) \
    X(256, 256, 64, 2, 2, 32, 2, 4654, 4525) \
    X(256, 256, 32, 2, 4, 32, 4, 2101, 2173) \
    X(256, 256, 32, 2, 2, 32, 4, 2224, 2287) \
    X(256, 256, 32, 2, 4, 32, 5, 2066, 2150) \
    X(256, 128, 64, 2, 4, 32, 3, 2415, 2468) \
    X(256, 128, 64, 2, 2, 32, 3, 2347, 2567) \
    X(128, 256, 64, 2, 4, 32, 3, 2340, 2392)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 2556, 2562) \
    X(128, 128, 64, 2, 2, 32, 2, 1192, 1190) \
    X(128, 128, 64, 2, 2, 32, 3, 1423, 1471) \
    X(64, 256, 64, 1, 4, 32, 2, 1442, 1357) \
    X(128, 64, 64, 2, 2, 32, 3, 762, 752) \
    X(64, 128, 64, 2, 2, 32, 3, 831, 750)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 524, 472) \
    X(64, 64, 128, 2, 2, 32, 2, 916, 911) \
    X(128, 32, 64, 4, 1, 32, 3, 627, 565) \
    X(32, 256, 64, 1, 4, 32, 2, 946, 933) \
    X(32, 128, 64, 1, 4, 32, 3, 555, 537) \
    X(32, 128, 128, 1, 4, 32, 2, 1038, 1033) \
    X(32, 64, 128, 1, 2, 32, 3, 635, 669)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 947, 1096) \
    X(16, 256, 128, 1, 4, 16, 2, 2286, 2225) \
    X(16, 128, 128, 1, 4, 16, 4, 1086, 1167) \
    X(16, 128, 256, 1, 4, 16, 2, 2526, 2462) \
    X(16, 64, 128, 1, 4, 16, 4, 455, 474) \
    X(16, 64, 256, 1, 4, 16, 3, 1341, 1395) \
    X(16, 32, 256, 1, 2, 16, 3, 844, 760) \
    X(16, 16, 256, 1, 1, 16, 3, 819, 737)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 4141, 4083) \
    X(256, 256, 64, 4, 2, 16, 2, 4044, 4026) \
    X(256, 128, 64, 2, 4, 16, 3, 2236, 2327) \
    X(128, 256, 64, 2, 4, 16, 3, 2202, 2340) \
    X(128, 128, 64, 2, 4, 16, 2, 1203, 1158) \
    X(128, 64, 64, 2, 4, 16, 3, 775, 738) \
    X(64, 128, 64, 2, 4, 16, 3, 746, 714) \
    X(128, 64, 64, 2, 4, 16, 2, 800, 766) \
    X(64, 128, 64, 2, 4, 16, 2, 918, 826) \
    X(64, 64, 64, 2, 4, 16, 3, 481, 453) \
    X(64, 64, 128, 2, 4, 16, 2, 927, 916) \
    X(128, 128, 64, 4, 2, 16, 2, 1218, 1149) \
    X(32, 64, 128, 1, 4, 16, 3, 621, 617)

// deeper LDS rings of tiles that win latency- and bandwidth-bound shapes (a request has NS-1 whole slabs
// of time to land); of eight such candidates these three were sweep-best on 10-20 % of the irregular shapes
#define G355_VARIANTS_BF16_5(X)    \
    X(64, 128, 64, 2, 4, 16, 4, 868, 868) \
    X(128, 128, 64, 2, 4, 16, 3, 1313, 1337) \
    X(128, 128, 64, 2, 4, 16, 4, 1323, 1314)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4373, 4254) \
    X(256, 256, 128, 2, 2, 32, 2, 4515, 4196) \
    X(256, 128, 128, 2, 4, 32, 3, 2304, 2350) \
    X(128, 256, 128, 2, 4, 32, 3, 2231, 2280) \
    X(128, 128, 128, 2, 2, 32, 2, 1125, 1143) \
    X(128, 128, 128, 2, 2, 32, 3, 1363, 1436) \
    X(128, 128, 256, 2, 2, 32, 2, 2865, 2866) \
    X(128, 64, 128, 2, 2, 32, 3, 842, 757) \
    X(64, 128, 128, 2, 2, 32, 3, 738, 749)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 1954, 1943) \
    X(64, 64, 128, 2, 2, 32, 3, 572, 514) \
    X(64, 64, 256, 2, 2, 32, 2, 1132, 1019) \
    X(64, 256, 128, 1, 4, 32, 2, 1216, 1263) \
    X(32, 256, 128, 1, 4, 32, 2, 959, 959) \
    X(32, 128, 256, 1, 4, 32, 2, 1058, 1087) \
    X(32, 32, 256, 1, 1, 32, 3, 800, 720) \
    X(16, 256, 256, 1, 4, 16, 2, 2634, 2536) \
    X(16, 128, 256, 1, 4, 16, 4, 1192, 1223) \
    X(16, 64, 256, 1, 4, 16, 4, 753, 678) \
    X(16, 16, 256, 1, 1, 16, 4, 669, 602)

#define G355_VARIANTS_BF16(X) \
    G355_VARIANTS_BF16_0(X) G355_VARIANTS_BF16_1(X) G355_VARIANTS_BF16_2(X) G355_VARIANTS_BF16_3(X) G355_VARIANTS_BF16_4(X) \
    G355_VARIANTS_BF16_5(X)
#define G355_VARIANTS_FP8(X) G355_VARIANTS_FP8_0(X) G355_VARIANTS_FP8_1(X)

namespace g355 {
struct Variant {
    int block_m, block_n, block_k, waves_m, waves_n, mfma, stages;
    int slab_clk;     // B row-major
    int slab_clk_kc;  // B K-contiguous
};
// Spatial K-unroll factors offered with every variant.
constexpr int kSplitKs[] = {1, 2, 4, 8, 16, 32};
constexpr int kNumSplitKs = sizeof(kSplitKs) / sizeof(kSplitKs[0]);
// Work splits offered with every variant: the split-K factors, then stream-K.
constexpr int kNumSplits = kNumSplitKs + 1;
inline int split_k_of(int mode) { return mode < kNumSplitKs ? kSplitKs[mode] : 1; }
inline int stream_k_of(int mode) { return mode == kNumSplitKs ? 1 : 0; }
}  // namespace g355
