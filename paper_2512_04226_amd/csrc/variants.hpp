// The compiled kernel variants: the candidate tile list the selector ranks (Section V-B of
// the paper speaks of 75 searched configurations; Section V-E of 50-150 valid tiles per
// datatype).  One line per instantiation of gemm_kernel<>:
//   X(BLOCK_M, BLOCK_N, BLOCK_K, WAVES_M, WAVES_N, MFMA, LDS_STAGES, SLAB_CLK, SLAB_CLK_KC, LOOP, LOOP_KC)
// LOOP / LOOP_KC: the K-loop form (0 to 3, see Tile in gemm_kernel.hpp) the instantiation for
// row-major / K-contiguous B is compiled with: the fastest of the four on 8192^3 where one is
// at least 1.5 % faster than form 0 (bf16 and fp16 timings together for the 16-bit list), else 0.
// SLAB_CLK (B row-major) and SLAB_CLK_KC (B K-contiguous; floored at 0.9 x SLAB_CLK, because the
// larger steady-state gains of the small tiles do not carry over to the small problems that
// use them) are calibration constants of the kernel, measured once on the device like the
// matrix-instruction latency L_MI: 2.4 GHz clocks a CU needs per K_T slab of one workgroup tile
// in steady state (all CUs busy, as many workgroups resident as fit), from an 8192^3 run.
// The order is part of the ABI of kernel_id and of the selector's tie-break (earlier wins).
#pragma once

// bf16: BLOCK_K in elements; MFMA 32 -> v_mfma_f32_32x32x16_bf16, 16 -> v_mfma_f32_16x16x32_bf16
#define G355_VARIANTS_BF16_0(X)    \
    X(256, 256, 64, 2, 4, 32, 2, 3794, 3870, 3, 3) \
    X(256, 256, 64, 2, 2, 32, 2, 4061, 4126, 3, 3) \
    X(256, 256, 32, 2, 4, 32, 4, 1908, 2036, 3, 3) \
    X(256, 256, 32, 2, 2, 32, 4, 2061, 2118, 3, 3) \
    X(256, 256, 32, 2, 4, 32, 5, 1913, 2050, 3, 3) \
    X(256, 128, 64, 2, 4, 32, 3, 2197, 2306, 3, 3) \
    X(256, 128, 64, 2, 2, 32, 3, 2339, 2415, 3, 3) \
    X(128, 256, 64, 2, 4, 32, 3, 2108, 2245, 3, 1)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 2336, 2381, 3, 3) \
    X(128, 128, 64, 2, 2, 32, 2, 1189, 1164, 0, 0) \
    X(128, 128, 64, 2, 2, 32, 3, 1321, 1382, 3, 1) \
    X(64, 256, 64, 1, 4, 32, 2, 1388, 1350, 1, 0) \
    X(128, 64, 64, 2, 2, 32, 3, 750, 723, 0, 3) \
    X(64, 128, 64, 2, 2, 32, 3, 725, 723, 1, 3)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 590, 531, 3, 0) \
    X(64, 64, 128, 2, 2, 32, 2, 918, 911, 0, 0) \
    X(128, 32, 64, 4, 1, 32, 3, 627, 564, 0, 0) \
    X(32, 256, 64, 1, 4, 32, 2, 940, 932, 2, 0) \
    X(32, 128, 64, 1, 4, 32, 3, 558, 532, 0, 0) \
    X(32, 128, 128, 1, 4, 32, 2, 1065, 1018, 0, 0) \
    X(32, 64, 128, 1, 2, 32, 3, 603, 622, 3, 1)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 867, 974, 3, 3) \
    X(16, 256, 128, 1, 4, 16, 2, 2270, 2186, 0, 3) \
    X(16, 128, 128, 1, 4, 16, 4, 972, 1008, 3, 3) \
    X(16, 128, 256, 1, 4, 16, 2, 2328, 2290, 3, 3) \
    X(16, 64, 128, 1, 4, 16, 4, 462, 481, 0, 0) \
    X(16, 64, 256, 1, 4, 16, 3, 1274, 1289, 3, 1) \
    X(16, 32, 256, 1, 2, 16, 3, 835, 751, 0, 1) \
    X(16, 16, 256, 1, 1, 16, 3, 819, 737, 0, 2)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 3789, 3796, 2, 2) \
    X(256, 256, 64, 4, 2, 16, 2, 3839, 3740, 2, 2) \
    X(256, 128, 64, 2, 4, 16, 3, 2055, 2089, 3, 3) \
    X(128, 256, 64, 2, 4, 16, 3, 2031, 2109, 1, 3) \
    X(128, 128, 64, 2, 4, 16, 2, 1179, 1138, 2, 0) \
    X(128, 64, 64, 2, 4, 16, 3, 757, 745, 3, 0) \
    X(64, 128, 64, 2, 4, 16, 3, 756, 706, 0, 1) \
    X(128, 64, 64, 2, 4, 16, 2, 775, 798, 0, 1) \
    X(64, 128, 64, 2, 4, 16, 2, 787, 740, 0, 0) \
    X(64, 64, 64, 2, 4, 16, 3, 478, 455, 0, 0) \
    X(64, 64, 128, 2, 4, 16, 2, 914, 925, 2, 0) \
    X(128, 128, 64, 4, 2, 16, 2, 1164, 1140, 1, 0) \
    X(32, 64, 128, 1, 4, 16, 3, 630, 609, 0, 3)

// deeper LDS rings of tiles that win latency- and bandwidth-bound shapes (a request has NS-1 whole slabs
// of time to land); of eight such candidates these three were sweep-best on 10-20 % of the irregular shapes
#define G355_VARIANTS_BF16_5(X)    \
    X(64, 128, 64, 2, 4, 16, 4, 818, 854, 2, 2) \
    X(128, 128, 64, 2, 4, 16, 3, 1224, 1218, 3, 1) \
    X(128, 128, 64, 2, 4, 16, 4, 1207, 1215, 3, 1)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 3636, 3587, 2, 3) \
    X(256, 256, 128, 2, 2, 32, 2, 3795, 3780, 3, 3) \
    X(256, 128, 128, 2, 4, 32, 3, 2168, 2134, 1, 1) \
    X(128, 256, 128, 2, 4, 32, 3, 2115, 2073, 3, 3) \
    X(128, 128, 128, 2, 2, 32, 2, 1066, 1090, 0, 0) \
    X(128, 128, 128, 2, 2, 32, 3, 1286, 1324, 3, 3) \
    X(128, 128, 256, 2, 2, 32, 2, 2748, 2775, 3, 0) \
    X(128, 64, 128, 2, 2, 32, 3, 817, 735, 0, 0) \
    X(64, 128, 128, 2, 2, 32, 3, 722, 730, 0, 2)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 1867, 1836, 3, 3) \
    X(64, 64, 128, 2, 2, 32, 3, 549, 494, 0, 1) \
    X(64, 64, 256, 2, 2, 32, 2, 1152, 1037, 0, 3) \
    X(64, 256, 128, 1, 4, 32, 2, 1201, 1188, 0, 0) \
    X(32, 256, 128, 1, 4, 32, 2, 963, 957, 0, 0) \
    X(32, 128, 256, 1, 4, 32, 2, 1101, 1059, 0, 3) \
    X(32, 32, 256, 1, 1, 32, 3, 791, 712, 0, 2) \
    X(16, 256, 256, 1, 4, 16, 2, 2568, 2492, 1, 0) \
    X(16, 128, 256, 1, 4, 16, 4, 1137, 1024, 3, 3) \
    X(16, 64, 256, 1, 4, 16, 4, 752, 677, 0, 1) \
    X(16, 16, 256, 1, 1, 16, 4, 669, 602, 0, 1)

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
