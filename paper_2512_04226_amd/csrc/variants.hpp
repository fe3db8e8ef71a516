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
    X(256, 256, 64, 2, 4, 32, 2, 5020, 4286) \
    X(256, 256, 64, 2, 2, 32, 2, 5610, 4390) \
    X(256, 256, 32, 2, 4, 32, 4, 2606, 2018) \
    X(256, 256, 32, 2, 2, 32, 4, 2912, 2267) \
    X(256, 256, 32, 2, 4, 32, 5, 2611, 2023) \
    X(256, 128, 64, 2, 4, 32, 3, 3114, 2343) \
    X(256, 128, 64, 2, 2, 32, 3, 3474, 2367) \
    X(128, 256, 64, 2, 4, 32, 3, 3152, 2212)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 3637, 2370) \
    X(128, 128, 64, 2, 2, 32, 2, 1370, 1112) \
    X(128, 128, 64, 2, 2, 32, 3, 2080, 1327) \
    X(128, 128, 128, 2, 2, 32, 2, 3381, 2705) \
    X(128, 128, 32, 2, 2, 32, 4, 885, 729) \
    X(256, 64, 64, 4, 1, 32, 2, 1447, 1263) \
    X(64, 256, 64, 1, 4, 32, 2, 1559, 1390) \
    X(128, 64, 64, 2, 2, 32, 3, 874, 716) \
    X(64, 128, 64, 2, 2, 32, 3, 886, 711)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 531, 444) \
    X(64, 64, 128, 2, 2, 32, 2, 1003, 878) \
    X(128, 32, 64, 4, 1, 32, 3, 725, 530) \
    X(32, 256, 64, 1, 4, 32, 2, 1033, 929) \
    X(32, 128, 64, 1, 4, 32, 3, 710, 526) \
    X(32, 128, 128, 1, 4, 32, 2, 1092, 1056) \
    X(32, 64, 128, 1, 2, 32, 3, 855, 615) \
    X(64, 32, 128, 2, 1, 32, 3, 909, 593) \
    X(32, 32, 128, 1, 1, 32, 3, 603, 383)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 1688, 879) \
    X(16, 256, 128, 1, 4, 16, 2, 2733, 2198) \
    X(16, 128, 128, 1, 4, 16, 4, 1728, 963) \
    X(16, 128, 256, 1, 4, 16, 2, 2954, 2303) \
    X(16, 64, 128, 1, 4, 16, 4, 664, 467) \
    X(16, 64, 256, 1, 4, 16, 3, 2056, 1257) \
    X(16, 32, 256, 1, 2, 16, 3, 997, 587) \
    X(16, 16, 256, 1, 1, 16, 3, 847, 389)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 4300, 3964) \
    X(256, 256, 64, 4, 2, 16, 2, 4689, 3978) \
    X(256, 128, 64, 2, 4, 16, 3, 2890, 2239) \
    X(128, 256, 64, 2, 4, 16, 3, 3065, 2163) \
    X(128, 128, 64, 2, 4, 16, 2, 1265, 1128) \
    X(128, 64, 64, 2, 4, 16, 3, 872, 737) \
    X(64, 128, 64, 2, 4, 16, 3, 849, 705) \
    X(128, 64, 64, 2, 4, 16, 2, 824, 817) \
    X(64, 128, 64, 2, 4, 16, 2, 784, 729) \
    X(64, 64, 64, 2, 4, 16, 3, 536, 447) \
    X(64, 64, 128, 2, 4, 16, 2, 1017, 915) \
    X(128, 128, 64, 4, 2, 16, 2, 1294, 1115) \
    X(32, 64, 128, 1, 4, 16, 3, 781, 598)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4601, 4238) \
    X(256, 256, 128, 2, 2, 32, 2, 5758, 4236) \
    X(256, 128, 128, 2, 4, 32, 3, 2669, 2322) \
    X(128, 256, 128, 2, 4, 32, 3, 2504, 2217) \
    X(128, 128, 128, 2, 2, 32, 2, 1168, 1084) \
    X(128, 128, 128, 2, 2, 32, 3, 2020, 1365) \
    X(128, 128, 256, 2, 2, 32, 2, 3471, 2845) \
    X(128, 64, 128, 2, 2, 32, 3, 909, 741) \
    X(64, 128, 128, 2, 2, 32, 3, 854, 743)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 2622, 1772) \
    X(64, 64, 128, 2, 2, 32, 3, 576, 470) \
    X(64, 64, 256, 2, 2, 32, 2, 1229, 933) \
    X(64, 256, 128, 1, 4, 32, 2, 1317, 1766) \
    X(32, 256, 128, 1, 4, 32, 2, 1025, 928) \
    X(32, 128, 256, 1, 4, 32, 2, 1144, 1075) \
    X(32, 32, 256, 1, 1, 32, 3, 979, 412) \
    X(16, 256, 256, 1, 4, 16, 2, 2926, 2548) \
    X(16, 128, 256, 1, 4, 16, 4, 1863, 1114) \
    X(16, 64, 256, 1, 4, 16, 4, 921, 493) \
    X(16, 16, 256, 1, 1, 16, 4, 684, 196)

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
