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
    X(256, 256, 64, 2, 4, 32, 2, 4637, 4181) \
    X(256, 256, 64, 2, 2, 32, 2, 4508, 4383) \
    X(256, 256, 32, 2, 4, 32, 4, 2064, 2109) \
    X(256, 256, 32, 2, 2, 32, 4, 2118, 2196) \
    X(256, 256, 32, 2, 4, 32, 5, 2035, 2119) \
    X(256, 128, 64, 2, 4, 32, 3, 2383, 2475) \
    X(256, 128, 64, 2, 2, 32, 3, 2338, 2515) \
    X(128, 256, 64, 2, 4, 32, 3, 2313, 2344)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 2535, 2627) \
    X(128, 128, 64, 2, 2, 32, 2, 1187, 1159) \
    X(128, 128, 64, 2, 2, 32, 3, 1408, 1435) \
    X(64, 256, 64, 1, 4, 32, 2, 1442, 1338) \
    X(128, 64, 64, 2, 2, 32, 3, 758, 747) \
    X(64, 128, 64, 2, 2, 32, 3, 850, 765)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 513, 462) \
    X(64, 64, 128, 2, 2, 32, 2, 902, 900) \
    X(128, 32, 64, 4, 1, 32, 3, 642, 578) \
    X(32, 256, 64, 1, 4, 32, 2, 918, 933) \
    X(32, 128, 64, 1, 4, 32, 3, 559, 532) \
    X(32, 128, 128, 1, 4, 32, 2, 1003, 1013) \
    X(32, 64, 128, 1, 2, 32, 3, 628, 659)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 950, 1091) \
    X(16, 256, 128, 1, 4, 16, 2, 2272, 2222) \
    X(16, 128, 128, 1, 4, 16, 4, 1072, 1096) \
    X(16, 128, 256, 1, 4, 16, 2, 2527, 2428) \
    X(16, 64, 128, 1, 4, 16, 4, 458, 475) \
    X(16, 64, 256, 1, 4, 16, 3, 1340, 1435) \
    X(16, 32, 256, 1, 2, 16, 3, 837, 754) \
    X(16, 16, 256, 1, 1, 16, 3, 820, 738)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 4136, 4041) \
    X(256, 256, 64, 4, 2, 16, 2, 4098, 3969) \
    X(256, 128, 64, 2, 4, 16, 3, 2260, 2311) \
    X(128, 256, 64, 2, 4, 16, 3, 2203, 2270) \
    X(128, 128, 64, 2, 4, 16, 2, 1206, 1133) \
    X(128, 64, 64, 2, 4, 16, 3, 769, 732) \
    X(64, 128, 64, 2, 4, 16, 3, 782, 705) \
    X(128, 64, 64, 2, 4, 16, 2, 796, 791) \
    X(64, 128, 64, 2, 4, 16, 2, 772, 736) \
    X(64, 64, 64, 2, 4, 16, 3, 488, 451) \
    X(64, 64, 128, 2, 4, 16, 2, 918, 921) \
    X(128, 128, 64, 4, 2, 16, 2, 1215, 1130) \
    X(32, 64, 128, 1, 4, 16, 3, 630, 619)

// deeper LDS rings of tiles that win latency- and bandwidth-bound shapes (a request has NS-1 whole slabs
// of time to land); of eight such candidates these three were sweep-best on 10-20 % of the irregular shapes
#define G355_VARIANTS_BF16_5(X)    \
    X(64, 128, 64, 2, 4, 16, 4, 820, 860) \
    X(128, 128, 64, 2, 4, 16, 3, 1306, 1294) \
    X(128, 128, 64, 2, 4, 16, 4, 1307, 1292)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4058, 4005) \
    X(256, 256, 128, 2, 2, 32, 2, 4043, 4032) \
    X(256, 128, 128, 2, 4, 32, 3, 2226, 2263) \
    X(128, 256, 128, 2, 4, 32, 3, 2152, 2199) \
    X(128, 128, 128, 2, 2, 32, 2, 1063, 1082) \
    X(128, 128, 128, 2, 2, 32, 3, 1314, 1312) \
    X(128, 128, 256, 2, 2, 32, 2, 2686, 2719) \
    X(128, 64, 128, 2, 2, 32, 3, 816, 734) \
    X(64, 128, 128, 2, 2, 32, 3, 715, 717)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 1918, 1945) \
    X(64, 64, 128, 2, 2, 32, 3, 556, 500) \
    X(64, 64, 256, 2, 2, 32, 2, 1134, 1020) \
    X(64, 256, 128, 1, 4, 32, 2, 1166, 1203) \
    X(32, 256, 128, 1, 4, 32, 2, 943, 952) \
    X(32, 128, 256, 1, 4, 32, 2, 1061, 1072) \
    X(32, 32, 256, 1, 1, 32, 3, 789, 710) \
    X(16, 256, 256, 1, 4, 16, 2, 2613, 2490) \
    X(16, 128, 256, 1, 4, 16, 4, 1185, 1209) \
    X(16, 64, 256, 1, 4, 16, 4, 751, 676) \
    X(16, 16, 256, 1, 1, 16, 4, 668, 601)

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
