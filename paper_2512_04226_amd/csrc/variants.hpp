// The compiled kernel variants: the candidate tile list the selector ranks (Section V-B of
// the paper speaks of 75 searched configurations; Section V-E of 50-150 valid tiles per
// datatype).  One line per instantiation of gemm_kernel<>:
//   X(BLOCK_M, BLOCK_N, BLOCK_K, WAVES_M, WAVES_N, MFMA, LDS_STAGES, SLAB_CLK, SLAB_CLK_KC)
// SLAB_CLK (B row-major) and SLAB_CLK_KC (B K-contiguous) are calibration constants of the
// kernel, measured once on the device like the
// matrix-instruction latency L_MI: 2.4 GHz clocks a CU needs per K_T slab of one workgroup tile
// in steady state (all CUs busy, as many workgroups resident as fit), from an 8192^3 run.
// The order is part of the ABI of kernel_id and of the selector's tie-break (earlier wins).
#pragma once

// bf16: BLOCK_K in elements; MFMA 32 -> v_mfma_f32_32x32x16_bf16, 16 -> v_mfma_f32_16x16x32_bf16
#define G355_VARIANTS_BF16_0(X)    \
    X(256, 256, 64, 2, 4, 32, 2, 5143, 4344) \
    X(256, 256, 64, 2, 2, 32, 2, 5212, 4282) \
    X(256, 256, 32, 2, 4, 32, 4, 2726, 2130) \
    X(256, 256, 32, 2, 2, 32, 4, 2974, 2216) \
    X(256, 256, 32, 2, 4, 32, 5, 2740, 2122) \
    X(256, 128, 64, 2, 4, 32, 3, 3159, 2327) \
    X(256, 128, 64, 2, 2, 32, 3, 3428, 2437) \
    X(128, 256, 64, 2, 4, 32, 3, 3162, 2277)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 3415, 2429) \
    X(128, 128, 64, 2, 2, 32, 2, 1356, 1175) \
    X(128, 128, 64, 2, 2, 32, 3, 2072, 1381) \
    X(128, 128, 128, 2, 2, 32, 2, 3445, 2802) \
    X(128, 128, 32, 2, 2, 32, 4, 913, 728) \
    X(256, 64, 64, 4, 1, 32, 2, 1432, 1308) \
    X(64, 256, 64, 1, 4, 32, 2, 1560, 1382) \
    X(128, 64, 64, 2, 2, 32, 3, 894, 716) \
    X(64, 128, 64, 2, 2, 32, 3, 890, 713)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 545, 447) \
    X(64, 64, 128, 2, 2, 32, 2, 1013, 872) \
    X(128, 32, 64, 4, 1, 32, 3, 750, 523) \
    X(32, 256, 64, 1, 4, 32, 2, 1057, 956) \
    X(32, 128, 64, 1, 4, 32, 3, 746, 532) \
    X(32, 128, 128, 1, 4, 32, 2, 1137, 1005) \
    X(32, 64, 128, 1, 2, 32, 3, 870, 595) \
    X(64, 32, 128, 2, 1, 32, 3, 887, 576) \
    X(32, 32, 128, 1, 1, 32, 3, 586, 374)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 1718, 896) \
    X(16, 256, 128, 1, 4, 16, 2, 2854, 2083) \
    X(16, 128, 128, 1, 4, 16, 4, 1868, 1113) \
    X(16, 128, 256, 1, 4, 16, 2, 3277, 2333) \
    X(16, 64, 128, 1, 4, 16, 4, 680, 461) \
    X(16, 64, 256, 1, 4, 16, 3, 2194, 1270) \
    X(16, 32, 256, 1, 2, 16, 3, 998, 579) \
    X(16, 16, 256, 1, 1, 16, 3, 794, 356)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4706, 4180) \
    X(256, 256, 128, 2, 2, 32, 2, 4913, 4183) \
    X(256, 128, 128, 2, 4, 32, 3, 2701, 2386) \
    X(128, 256, 128, 2, 4, 32, 3, 2510, 2239) \
    X(128, 128, 128, 2, 2, 32, 2, 1197, 1126) \
    X(128, 128, 128, 2, 2, 32, 3, 1995, 1419) \
    X(128, 128, 256, 2, 2, 32, 2, 3550, 2779) \
    X(128, 64, 128, 2, 2, 32, 3, 907, 732) \
    X(64, 128, 128, 2, 2, 32, 3, 845, 731)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 2599, 1826) \
    X(64, 64, 128, 2, 2, 32, 3, 604, 470) \
    X(64, 64, 256, 2, 2, 32, 2, 1221, 922) \
    X(64, 256, 128, 1, 4, 32, 2, 1308, 1245) \
    X(32, 256, 128, 1, 4, 32, 2, 1043, 910) \
    X(32, 128, 256, 1, 4, 32, 2, 1139, 1036) \
    X(32, 32, 256, 1, 1, 32, 3, 823, 385) \
    X(16, 256, 256, 1, 4, 16, 2, 3058, 2371) \
    X(16, 128, 256, 1, 4, 16, 4, 1951, 1123) \
    X(16, 64, 256, 1, 4, 16, 4, 944, 483) \
    X(16, 16, 256, 1, 1, 16, 4, 675, 177)

#define G355_VARIANTS_BF16(X) G355_VARIANTS_BF16_0(X) G355_VARIANTS_BF16_1(X) G355_VARIANTS_BF16_2(X) G355_VARIANTS_BF16_3(X)
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
