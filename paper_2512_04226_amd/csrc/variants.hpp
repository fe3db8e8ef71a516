// The compiled kernel variants: the candidate tile list the selector ranks (Section V-B of
// the paper speaks of 75 searched configurations; Section V-E of 50-150 valid tiles per
// datatype).  One line per instantiation of gemm_kernel<>:
//   X(BLOCK_M, BLOCK_N, BLOCK_K, WAVES_M, WAVES_N, MFMA, LDS_STAGES, SLAB_CLK, SLAB_CLK_KC, LOOP, LOOP_KC)
// LOOP / LOOP_KC: the K-loop form (0, 1 or 2, see Tile in gemm_kernel.hpp) the instantiation for
// row-major / K-contiguous B is compiled with: the fastest of the three on 8192^3 where one is
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
    X(256, 256, 64, 2, 4, 32, 2, 4046, 4015, 2, 1) \
    X(256, 256, 64, 2, 2, 32, 2, 4353, 4318, 0, 1) \
    X(256, 256, 32, 2, 4, 32, 4, 2021, 2139, 1, 2) \
    X(256, 256, 32, 2, 2, 32, 4, 2158, 2236, 2, 1) \
    X(256, 256, 32, 2, 4, 32, 5, 2036, 2152, 1, 2) \
    X(256, 128, 64, 2, 4, 32, 3, 2288, 2382, 1, 1) \
    X(256, 128, 64, 2, 2, 32, 3, 2403, 2518, 0, 2) \
    X(128, 256, 64, 2, 4, 32, 3, 2205, 2295, 1, 1)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 2487, 2521, 2, 2) \
    X(128, 128, 64, 2, 2, 32, 2, 1204, 1195, 0, 0) \
    X(128, 128, 64, 2, 2, 32, 3, 1364, 1434, 1, 1) \
    X(64, 256, 64, 1, 4, 32, 2, 1355, 1358, 1, 0) \
    X(128, 64, 64, 2, 2, 32, 3, 759, 757, 1, 1) \
    X(64, 128, 64, 2, 2, 32, 3, 734, 763, 1, 0)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 501, 461, 0, 0) \
    X(64, 64, 128, 2, 2, 32, 2, 928, 926, 0, 0) \
    X(128, 32, 64, 4, 1, 32, 3, 649, 584, 0, 0) \
    X(32, 256, 64, 1, 4, 32, 2, 934, 947, 0, 0) \
    X(32, 128, 64, 1, 4, 32, 3, 562, 543, 0, 0) \
    X(32, 128, 128, 1, 4, 32, 2, 1038, 1041, 0, 0) \
    X(32, 64, 128, 1, 2, 32, 3, 634, 633, 2, 1)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 891, 996, 2, 1) \
    X(16, 256, 128, 1, 4, 16, 2, 2268, 2217, 0, 0) \
    X(16, 128, 128, 1, 4, 16, 4, 1070, 1089, 0, 0) \
    X(16, 128, 256, 1, 4, 16, 2, 2340, 2289, 1, 1) \
    X(16, 64, 128, 1, 4, 16, 4, 471, 488, 0, 0) \
    X(16, 64, 256, 1, 4, 16, 3, 1334, 1291, 0, 2) \
    X(16, 32, 256, 1, 2, 16, 3, 836, 752, 0, 2) \
    X(16, 16, 256, 1, 1, 16, 3, 819, 737, 0, 2)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 3845, 3857, 2, 2) \
    X(256, 256, 64, 4, 2, 16, 2, 3916, 3828, 1, 2) \
    X(256, 128, 64, 2, 4, 16, 3, 2290, 2288, 0, 1) \
    X(128, 256, 64, 2, 4, 16, 3, 2101, 2297, 1, 2) \
    X(128, 128, 64, 2, 4, 16, 2, 1180, 1153, 2, 0) \
    X(128, 64, 64, 2, 4, 16, 3, 796, 755, 0, 1) \
    X(64, 128, 64, 2, 4, 16, 3, 764, 729, 0, 0) \
    X(128, 64, 64, 2, 4, 16, 2, 790, 796, 0, 2) \
    X(64, 128, 64, 2, 4, 16, 2, 793, 758, 0, 0) \
    X(64, 64, 64, 2, 4, 16, 3, 482, 465, 2, 0) \
    X(64, 64, 128, 2, 4, 16, 2, 925, 936, 2, 0) \
    X(128, 128, 64, 4, 2, 16, 2, 1185, 1158, 2, 0) \
    X(32, 64, 128, 1, 4, 16, 3, 643, 634, 0, 0)

// deeper LDS rings of tiles that win latency- and bandwidth-bound shapes (a request has NS-1 whole slabs
// of time to land); of eight such candidates these three were sweep-best on 10-20 % of the irregular shapes
#define G355_VARIANTS_BF16_5(X)    \
    X(64, 128, 64, 2, 4, 16, 4, 846, 866, 2, 2) \
    X(128, 128, 64, 2, 4, 16, 3, 1310, 1247, 2, 1) \
    X(128, 128, 64, 2, 4, 16, 4, 1311, 1239, 2, 1)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 3743, 3933, 2, 0) \
    X(256, 256, 128, 2, 2, 32, 2, 4220, 4156, 0, 0) \
    X(256, 128, 128, 2, 4, 32, 3, 2233, 2163, 1, 1) \
    X(128, 256, 128, 2, 4, 32, 3, 2165, 2179, 1, 1) \
    X(128, 128, 128, 2, 2, 32, 2, 1109, 1120, 0, 0) \
    X(128, 128, 128, 2, 2, 32, 3, 1362, 1372, 0, 0) \
    X(128, 128, 256, 2, 2, 32, 2, 2833, 2819, 0, 0) \
    X(128, 64, 128, 2, 2, 32, 3, 837, 753, 0, 1) \
    X(64, 128, 128, 2, 2, 32, 3, 742, 743, 0, 0)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 1900, 1933, 0, 0) \
    X(64, 64, 128, 2, 2, 32, 3, 563, 506, 0, 2) \
    X(64, 64, 256, 2, 2, 32, 2, 1166, 1050, 0, 2) \
    X(64, 256, 128, 1, 4, 32, 2, 1205, 1231, 0, 0) \
    X(32, 256, 128, 1, 4, 32, 2, 979, 983, 0, 0) \
    X(32, 128, 256, 1, 4, 32, 2, 1130, 1108, 0, 0) \
    X(32, 32, 256, 1, 1, 32, 3, 780, 702, 1, 2) \
    X(16, 256, 256, 1, 4, 16, 2, 2565, 2489, 1, 0) \
    X(16, 128, 256, 1, 4, 16, 4, 1179, 1089, 0, 1) \
    X(16, 64, 256, 1, 4, 16, 4, 750, 675, 0, 1) \
    X(16, 16, 256, 1, 1, 16, 4, 664, 598, 0, 1)

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
