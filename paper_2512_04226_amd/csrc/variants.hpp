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
    X(256, 256, 64, 2, 4, 32, 2, 5074, 4299) \
    X(256, 256, 64, 2, 2, 32, 2, 5704, 4705) \
    X(256, 256, 32, 2, 4, 32, 4, 2655, 2216) \
    X(256, 256, 32, 2, 2, 32, 4, 2935, 2472) \
    X(256, 256, 32, 2, 4, 32, 5, 2638, 2219) \
    X(256, 128, 64, 2, 4, 32, 3, 3160, 2441) \
    X(256, 128, 64, 2, 2, 32, 3, 3490, 2479) \
    X(128, 256, 64, 2, 4, 32, 3, 3186, 2336)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 3635, 2490) \
    X(128, 128, 64, 2, 2, 32, 2, 1391, 1192) \
    X(128, 128, 64, 2, 2, 32, 3, 2086, 1387) \
    X(128, 128, 128, 2, 2, 32, 2, 3405, 2893) \
    X(128, 128, 32, 2, 2, 32, 4, 890, 756) \
    X(256, 64, 64, 4, 1, 32, 2, 1458, 1307) \
    X(64, 256, 64, 1, 4, 32, 2, 1567, 1432) \
    X(128, 64, 64, 2, 2, 32, 3, 895, 741) \
    X(64, 128, 64, 2, 2, 32, 3, 913, 742)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 546, 459) \
    X(64, 64, 128, 2, 2, 32, 2, 1034, 915) \
    X(128, 32, 64, 4, 1, 32, 3, 725, 539) \
    X(32, 256, 64, 1, 4, 32, 2, 1054, 978) \
    X(32, 128, 64, 1, 4, 32, 3, 710, 546) \
    X(32, 128, 128, 1, 4, 32, 2, 1138, 1077) \
    X(32, 64, 128, 1, 2, 32, 3, 855, 641) \
    X(64, 32, 128, 2, 1, 32, 3, 910, 624) \
    X(32, 32, 128, 1, 1, 32, 3, 602, 397)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 1687, 879) \
    X(16, 256, 128, 1, 4, 16, 2, 2735, 2199) \
    X(16, 128, 128, 1, 4, 16, 4, 1729, 964) \
    X(16, 128, 256, 1, 4, 16, 2, 2955, 2302) \
    X(16, 64, 128, 1, 4, 16, 4, 665, 481) \
    X(16, 64, 256, 1, 4, 16, 3, 2059, 1255) \
    X(16, 32, 256, 1, 2, 16, 3, 998, 587) \
    X(16, 16, 256, 1, 1, 16, 3, 865, 388) \
    X(256, 256, 64, 2, 4, 16, 2, 4441, 4090) \
    X(256, 256, 64, 4, 2, 16, 2, 4794, 4111) \
    X(256, 128, 64, 2, 4, 16, 3, 2911, 2340) \
    X(128, 256, 64, 2, 4, 16, 3, 3066, 2337) \
    X(128, 128, 64, 2, 4, 16, 2, 1302, 1161) \
    X(128, 64, 64, 2, 4, 16, 3, 887, 745) \
    X(64, 128, 64, 2, 4, 16, 3, 873, 731)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4770, 4306) \
    X(256, 256, 128, 2, 2, 32, 2, 5767, 4395) \
    X(256, 128, 128, 2, 4, 32, 3, 2758, 2451) \
    X(128, 256, 128, 2, 4, 32, 3, 2545, 2307) \
    X(128, 128, 128, 2, 2, 32, 2, 1233, 1122) \
    X(128, 128, 128, 2, 2, 32, 3, 2024, 1459) \
    X(128, 128, 256, 2, 2, 32, 2, 3489, 2893) \
    X(128, 64, 128, 2, 2, 32, 3, 933, 756) \
    X(64, 128, 128, 2, 2, 32, 3, 878, 754)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 2625, 1838) \
    X(64, 64, 128, 2, 2, 32, 3, 600, 490) \
    X(64, 64, 256, 2, 2, 32, 2, 1259, 961) \
    X(64, 256, 128, 1, 4, 32, 2, 1362, 1818) \
    X(32, 256, 128, 1, 4, 32, 2, 1049, 967) \
    X(32, 128, 256, 1, 4, 32, 2, 1165, 1119) \
    X(32, 32, 256, 1, 1, 32, 3, 978, 411) \
    X(16, 256, 256, 1, 4, 16, 2, 2924, 2545) \
    X(16, 128, 256, 1, 4, 16, 4, 1866, 1115) \
    X(16, 64, 256, 1, 4, 16, 4, 924, 506) \
    X(16, 16, 256, 1, 1, 16, 4, 684, 195)

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
