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
    X(256, 256, 64, 2, 4, 32, 2, 5036) \
    X(256, 256, 64, 2, 2, 32, 2, 5201) \
    X(256, 256, 32, 2, 4, 32, 4, 2737) \
    X(256, 256, 32, 2, 2, 32, 4, 2992) \
    X(256, 256, 32, 2, 4, 32, 5, 2715) \
    X(256, 128, 64, 2, 4, 32, 3, 3156) \
    X(256, 128, 64, 2, 2, 32, 3, 3428) \
    X(128, 256, 64, 2, 4, 32, 3, 3158)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 3397) \
    X(128, 128, 64, 2, 2, 32, 2, 1365) \
    X(128, 128, 64, 2, 2, 32, 3, 2079) \
    X(128, 128, 128, 2, 2, 32, 2, 3440) \
    X(128, 128, 32, 2, 2, 32, 4, 920) \
    X(256, 64, 64, 4, 1, 32, 2, 1452) \
    X(64, 256, 64, 1, 4, 32, 2, 1537) \
    X(128, 64, 64, 2, 2, 32, 3, 890) \
    X(64, 128, 64, 2, 2, 32, 3, 893)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 551) \
    X(64, 64, 128, 2, 2, 32, 2, 1013) \
    X(128, 32, 64, 4, 1, 32, 3, 753) \
    X(32, 256, 64, 1, 4, 32, 2, 1058) \
    X(32, 128, 64, 1, 4, 32, 3, 746) \
    X(32, 128, 128, 1, 4, 32, 2, 1124) \
    X(32, 64, 128, 1, 2, 32, 3, 871) \
    X(64, 32, 128, 2, 1, 32, 3, 887) \
    X(32, 32, 128, 1, 1, 32, 3, 587)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 1719) \
    X(16, 256, 128, 1, 4, 16, 2, 2857) \
    X(16, 128, 128, 1, 4, 16, 4, 1872) \
    X(16, 128, 256, 1, 4, 16, 2, 3277) \
    X(16, 64, 128, 1, 4, 16, 4, 680) \
    X(16, 64, 256, 1, 4, 16, 3, 2198) \
    X(16, 32, 256, 1, 2, 16, 3, 1000) \
    X(16, 16, 256, 1, 1, 16, 3, 798)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 4712) \
    X(256, 256, 128, 2, 2, 32, 2, 5001) \
    X(256, 128, 128, 2, 4, 32, 3, 2668) \
    X(128, 256, 128, 2, 4, 32, 3, 2461) \
    X(128, 128, 128, 2, 2, 32, 2, 1221) \
    X(128, 128, 128, 2, 2, 32, 3, 2005) \
    X(128, 128, 256, 2, 2, 32, 2, 3542) \
    X(128, 64, 128, 2, 2, 32, 3, 905) \
    X(64, 128, 128, 2, 2, 32, 3, 846)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 2602) \
    X(64, 64, 128, 2, 2, 32, 3, 587) \
    X(64, 64, 256, 2, 2, 32, 2, 1219) \
    X(64, 256, 128, 1, 4, 32, 2, 1293) \
    X(32, 256, 128, 1, 4, 32, 2, 1035) \
    X(32, 128, 256, 1, 4, 32, 2, 1144) \
    X(32, 32, 256, 1, 1, 32, 3, 831) \
    X(16, 256, 256, 1, 4, 16, 2, 3073) \
    X(16, 128, 256, 1, 4, 16, 4, 1954) \
    X(16, 64, 256, 1, 4, 16, 4, 943) \
    X(16, 16, 256, 1, 1, 16, 4, 674)

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
}  // namespace g355
