// The compiled kernel variants: the candidate tile list the selector ranks (Section V-B of
// the paper speaks of 75 searched configurations; Section V-E of 50-150 valid tiles per
// datatype).  One line per instantiation of gemm_kernel<>:
//   X(BLOCK_M, BLOCK_N, BLOCK_K, WAVES_M, WAVES_N, MFMA, LDS_STAGES, SLAB_CLK)
// SLAB_CLK is a calibration constant of the kernel, measured once on the device like the
// matrix-instruction latency L_MI: 2.4 GHz clocks a CU needs per K_T slab of one workgroup tile
// in steady state (all CUs busy, as many workgroups resident as fit), from an 8192^3 run.
// The order is part of the ABI of kernel_id and of the selector's tie-break (earlier wins).
#pragma once

// bf16: BLOCK_K in elements; MFMA 32 -> v_mfma_f32_32x32x16_bf16, 16 -> v_mfma_f32_16x16x32_bf16
#define G355_VARIANTS_BF16_0(X)    \
    X(256, 256, 64, 2, 4, 32, 2, 4691) \
    X(256, 256, 64, 2, 2, 32, 2, 5138) \
    X(256, 256, 32, 2, 4, 32, 4, 2787) \
    X(256, 256, 32, 2, 2, 32, 4, 2941) \
    X(256, 256, 32, 2, 4, 32, 5, 2769) \
    X(256, 128, 64, 2, 4, 32, 3, 3156) \
    X(256, 128, 64, 2, 2, 32, 3, 3435) \
    X(128, 256, 64, 2, 4, 32, 3, 3310)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 3524) \
    X(128, 128, 64, 2, 2, 32, 2, 1404) \
    X(128, 128, 64, 2, 2, 32, 3, 2130) \
    X(128, 128, 128, 2, 2, 32, 2, 3569) \
    X(128, 128, 32, 2, 2, 32, 4, 927) \
    X(256, 64, 64, 4, 1, 32, 2, 1524) \
    X(64, 256, 64, 1, 4, 32, 2, 1565) \
    X(128, 64, 64, 2, 2, 32, 3, 934) \
    X(64, 128, 64, 2, 2, 32, 3, 916)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 551) \
    X(64, 64, 128, 2, 2, 32, 2, 1040) \
    X(128, 32, 64, 4, 1, 32, 3, 763) \
    X(32, 256, 64, 1, 4, 32, 2, 1025) \
    X(32, 128, 64, 1, 4, 32, 3, 737) \
    X(32, 128, 128, 1, 4, 32, 2, 1154) \
    X(32, 64, 128, 1, 2, 32, 3, 881) \
    X(64, 32, 128, 2, 1, 32, 3, 906) \
    X(32, 32, 128, 1, 1, 32, 3, 621)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 1710) \
    X(16, 256, 128, 1, 4, 16, 2, 2663) \
    X(16, 128, 128, 1, 4, 16, 4, 1769) \
    X(16, 128, 256, 1, 4, 16, 2, 3138) \
    X(16, 64, 128, 1, 4, 16, 4, 641) \
    X(16, 64, 256, 1, 4, 16, 3, 2105) \
    X(16, 32, 256, 1, 2, 16, 3, 954) \
    X(16, 16, 256, 1, 1, 16, 3, 942)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4601) \
    X(256, 256, 128, 2, 2, 32, 2, 4995) \
    X(256, 128, 128, 2, 4, 32, 3, 2862) \
    X(128, 256, 128, 2, 4, 32, 3, 2875) \
    X(128, 128, 128, 2, 2, 32, 2, 1326) \
    X(128, 128, 128, 2, 2, 32, 3, 2175) \
    X(128, 128, 256, 2, 2, 32, 2, 3777) \
    X(128, 64, 128, 2, 2, 32, 3, 954) \
    X(64, 128, 128, 2, 2, 32, 3, 893)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 2893) \
    X(64, 64, 128, 2, 2, 32, 3, 585) \
    X(64, 64, 256, 2, 2, 32, 2, 1167) \
    X(64, 256, 128, 1, 4, 32, 2, 1420) \
    X(32, 256, 128, 1, 4, 32, 2, 1044) \
    X(32, 128, 256, 1, 4, 32, 2, 1182) \
    X(32, 32, 256, 1, 1, 32, 3, 883) \
    X(16, 256, 256, 1, 4, 16, 2, 2869) \
    X(16, 128, 256, 1, 4, 16, 4, 1815) \
    X(16, 64, 256, 1, 4, 16, 4, 893) \
    X(16, 16, 256, 1, 1, 16, 4, 669)

#define G355_VARIANTS_BF16(X) G355_VARIANTS_BF16_0(X) G355_VARIANTS_BF16_1(X) G355_VARIANTS_BF16_2(X) G355_VARIANTS_BF16_3(X)
#define G355_VARIANTS_FP8(X) G355_VARIANTS_FP8_0(X) G355_VARIANTS_FP8_1(X)

namespace g355 {
struct Variant {
    int block_m, block_n, block_k, waves_m, waves_n, mfma, stages, slab_clk;
};
// Spatial K-unroll factors offered with every variant.
constexpr int kSplitKs[] = {1, 2, 4, 8, 16, 32};
constexpr int kNumSplitKs = sizeof(kSplitKs) / sizeof(kSplitKs[0]);
}  // namespace g355
