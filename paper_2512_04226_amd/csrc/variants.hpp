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
    X(256, 256, 64, 2, 4, 32, 2, 5020, 4518) \
    X(256, 256, 64, 2, 2, 32, 2, 5610, 5049) \
    X(256, 256, 32, 2, 4, 32, 4, 2606, 2345) \
    X(256, 256, 32, 2, 2, 32, 4, 2912, 2621) \
    X(256, 256, 32, 2, 4, 32, 5, 2611, 2350) \
    X(256, 128, 64, 2, 4, 32, 3, 3114, 2803) \
    X(256, 128, 64, 2, 2, 32, 3, 3474, 3127) \
    X(128, 256, 64, 2, 4, 32, 3, 3152, 2837)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 3637, 3273) \
    X(128, 128, 64, 2, 2, 32, 2, 1370, 1233) \
    X(128, 128, 64, 2, 2, 32, 3, 2080, 1872) \
    X(128, 128, 128, 2, 2, 32, 2, 3381, 3043) \
    X(128, 128, 32, 2, 2, 32, 4, 885, 796) \
    X(256, 64, 64, 4, 1, 32, 2, 1447, 1302) \
    X(64, 256, 64, 1, 4, 32, 2, 1559, 1403) \
    X(128, 64, 64, 2, 2, 32, 3, 874, 787) \
    X(64, 128, 64, 2, 2, 32, 3, 886, 797)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 531, 478) \
    X(64, 64, 128, 2, 2, 32, 2, 1003, 903) \
    X(128, 32, 64, 4, 1, 32, 3, 725, 652) \
    X(32, 256, 64, 1, 4, 32, 2, 1033, 930) \
    X(32, 128, 64, 1, 4, 32, 3, 710, 639) \
    X(32, 128, 128, 1, 4, 32, 2, 1092, 1056) \
    X(32, 64, 128, 1, 2, 32, 3, 855, 770) \
    X(64, 32, 128, 2, 1, 32, 3, 909, 818) \
    X(32, 32, 128, 1, 1, 32, 3, 603, 543)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 1688, 1519) \
    X(16, 256, 128, 1, 4, 16, 2, 2733, 2460) \
    X(16, 128, 128, 1, 4, 16, 4, 1728, 1555) \
    X(16, 128, 256, 1, 4, 16, 2, 2954, 2659) \
    X(16, 64, 128, 1, 4, 16, 4, 664, 598) \
    X(16, 64, 256, 1, 4, 16, 3, 2056, 1850) \
    X(16, 32, 256, 1, 2, 16, 3, 997, 897) \
    X(16, 16, 256, 1, 1, 16, 3, 847, 762)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 4300, 3964) \
    X(256, 256, 64, 4, 2, 16, 2, 4689, 4220) \
    X(256, 128, 64, 2, 4, 16, 3, 2890, 2601) \
    X(128, 256, 64, 2, 4, 16, 3, 3065, 2758) \
    X(128, 128, 64, 2, 4, 16, 2, 1265, 1138) \
    X(128, 64, 64, 2, 4, 16, 3, 872, 785) \
    X(64, 128, 64, 2, 4, 16, 3, 849, 764) \
    X(128, 64, 64, 2, 4, 16, 2, 824, 817) \
    X(64, 128, 64, 2, 4, 16, 2, 784, 729) \
    X(64, 64, 64, 2, 4, 16, 3, 536, 482) \
    X(64, 64, 128, 2, 4, 16, 2, 1017, 915) \
    X(128, 128, 64, 4, 2, 16, 2, 1294, 1165) \
    X(32, 64, 128, 1, 4, 16, 3, 781, 703)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4601, 4238) \
    X(256, 256, 128, 2, 2, 32, 2, 5758, 5182) \
    X(256, 128, 128, 2, 4, 32, 3, 2669, 2402) \
    X(128, 256, 128, 2, 4, 32, 3, 2504, 2254) \
    X(128, 128, 128, 2, 2, 32, 2, 1168, 1084) \
    X(128, 128, 128, 2, 2, 32, 3, 2020, 1818) \
    X(128, 128, 256, 2, 2, 32, 2, 3471, 3124) \
    X(128, 64, 128, 2, 2, 32, 3, 909, 818) \
    X(64, 128, 128, 2, 2, 32, 3, 854, 769)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 2622, 2360) \
    X(64, 64, 128, 2, 2, 32, 3, 576, 518) \
    X(64, 64, 256, 2, 2, 32, 2, 1229, 1106) \
    X(64, 256, 128, 1, 4, 32, 2, 1317, 1766) \
    X(32, 256, 128, 1, 4, 32, 2, 1025, 928) \
    X(32, 128, 256, 1, 4, 32, 2, 1144, 1075) \
    X(32, 32, 256, 1, 1, 32, 3, 979, 881) \
    X(16, 256, 256, 1, 4, 16, 2, 2926, 2633) \
    X(16, 128, 256, 1, 4, 16, 4, 1863, 1677) \
    X(16, 64, 256, 1, 4, 16, 4, 921, 829) \
    X(16, 16, 256, 1, 1, 16, 4, 684, 616)

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
