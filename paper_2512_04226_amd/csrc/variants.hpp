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
    X(256, 256, 64, 2, 4, 32, 2, 4810, 4329) \
    X(256, 256, 64, 2, 2, 32, 2, 4781, 4560) \
    X(256, 256, 32, 2, 4, 32, 4, 2155, 2184) \
    X(256, 256, 32, 2, 2, 32, 4, 2268, 2287) \
    X(256, 256, 32, 2, 4, 32, 5, 2115, 2172) \
    X(256, 128, 64, 2, 4, 32, 3, 2466, 2532) \
    X(256, 128, 64, 2, 2, 32, 3, 2399, 2691) \
    X(128, 256, 64, 2, 4, 32, 3, 2361, 2460)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 2557, 2635) \
    X(128, 128, 64, 2, 2, 32, 2, 1211, 1201) \
    X(128, 128, 64, 2, 2, 32, 3, 1447, 1509) \
    X(128, 128, 128, 2, 2, 32, 2, 3007, 3238) \
    X(128, 128, 32, 2, 2, 32, 4, 689, 750) \
    X(256, 64, 64, 4, 1, 32, 2, 1328, 1284) \
    X(64, 256, 64, 1, 4, 32, 2, 1471, 1373) \
    X(128, 64, 64, 2, 2, 32, 3, 770, 759) \
    X(64, 128, 64, 2, 2, 32, 3, 828, 761)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 576, 518) \
    X(64, 64, 128, 2, 2, 32, 2, 937, 939) \
    X(128, 32, 64, 4, 1, 32, 3, 638, 574) \
    X(32, 256, 64, 1, 4, 32, 2, 961, 953) \
    X(32, 128, 64, 1, 4, 32, 3, 564, 547) \
    X(32, 128, 128, 1, 4, 32, 2, 1064, 1044) \
    X(32, 64, 128, 1, 2, 32, 3, 660, 681) \
    X(64, 32, 128, 2, 1, 32, 3, 726, 695) \
    X(32, 32, 128, 1, 1, 32, 3, 526, 474)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 948, 1100) \
    X(16, 256, 128, 1, 4, 16, 2, 2288, 2226) \
    X(16, 128, 128, 1, 4, 16, 4, 1087, 1166) \
    X(16, 128, 256, 1, 4, 16, 2, 2528, 2465) \
    X(16, 64, 128, 1, 4, 16, 4, 461, 482) \
    X(16, 64, 256, 1, 4, 16, 3, 1341, 1397) \
    X(16, 32, 256, 1, 2, 16, 3, 842, 758) \
    X(16, 16, 256, 1, 1, 16, 3, 819, 737)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 4228, 4161) \
    X(256, 256, 64, 4, 2, 16, 2, 4148, 4092) \
    X(256, 128, 64, 2, 4, 16, 3, 2350, 2384) \
    X(128, 256, 64, 2, 4, 16, 3, 2280, 2345) \
    X(128, 128, 64, 2, 4, 16, 2, 1243, 1165) \
    X(128, 64, 64, 2, 4, 16, 3, 779, 747) \
    X(64, 128, 64, 2, 4, 16, 3, 745, 727) \
    X(128, 64, 64, 2, 4, 16, 2, 804, 768) \
    X(64, 128, 64, 2, 4, 16, 2, 918, 826) \
    X(64, 64, 64, 2, 4, 16, 3, 490, 457) \
    X(64, 64, 128, 2, 4, 16, 2, 951, 938) \
    X(128, 128, 64, 4, 2, 16, 2, 1238, 1165) \
    X(32, 64, 128, 1, 4, 16, 3, 644, 637)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4420, 4241) \
    X(256, 256, 128, 2, 2, 32, 2, 4584, 4150) \
    X(256, 128, 128, 2, 4, 32, 3, 2370, 2392) \
    X(128, 256, 128, 2, 4, 32, 3, 2294, 2335) \
    X(128, 128, 128, 2, 2, 32, 2, 1139, 1150) \
    X(128, 128, 128, 2, 2, 32, 3, 1422, 1472) \
    X(128, 128, 256, 2, 2, 32, 2, 2988, 2990) \
    X(128, 64, 128, 2, 2, 32, 3, 847, 763) \
    X(64, 128, 128, 2, 2, 32, 3, 746, 756)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 1962, 1942) \
    X(64, 64, 128, 2, 2, 32, 3, 578, 520) \
    X(64, 64, 256, 2, 2, 32, 2, 1144, 1030) \
    X(64, 256, 128, 1, 4, 32, 2, 1230, 1297) \
    X(32, 256, 128, 1, 4, 32, 2, 974, 983) \
    X(32, 128, 256, 1, 4, 32, 2, 1082, 1123) \
    X(32, 32, 256, 1, 1, 32, 3, 803, 722) \
    X(16, 256, 256, 1, 4, 16, 2, 2633, 2537) \
    X(16, 128, 256, 1, 4, 16, 4, 1192, 1223) \
    X(16, 64, 256, 1, 4, 16, 4, 756, 680) \
    X(16, 16, 256, 1, 1, 16, 4, 669, 602)

#define G355_VARIANTS_BF16(X) \
    G355_VARIANTS_BF16_0(X) G355_VARIANTS_BF16_1(X) G355_VARIANTS_BF16_2(X) G355_VARIANTS_BF16_3(X) G355_VARIANTS_BF16_4(X)
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
