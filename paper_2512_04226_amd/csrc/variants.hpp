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
    X(256, 256, 64, 2, 4, 32, 2, 4062, 4208) \
    X(256, 256, 64, 2, 2, 32, 2, 4334, 4495) \
    X(256, 256, 32, 2, 4, 32, 4, 2070, 2139) \
    X(256, 256, 32, 2, 2, 32, 4, 2170, 2267) \
    X(256, 256, 32, 2, 4, 32, 5, 2074, 2167) \
    X(256, 128, 64, 2, 4, 32, 3, 2418, 2489) \
    X(256, 128, 64, 2, 2, 32, 3, 2392, 2583) \
    X(128, 256, 64, 2, 4, 32, 3, 2361, 2385)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 2588, 2719) \
    X(128, 128, 64, 2, 2, 32, 2, 1198, 1185) \
    X(128, 128, 64, 2, 2, 32, 3, 1440, 1472) \
    X(64, 256, 64, 1, 4, 32, 2, 1430, 1357) \
    X(128, 64, 64, 2, 2, 32, 3, 763, 758) \
    X(64, 128, 64, 2, 2, 32, 3, 845, 761)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 601, 541) \
    X(64, 64, 128, 2, 2, 32, 2, 924, 925) \
    X(128, 32, 64, 4, 1, 32, 3, 622, 559) \
    X(32, 256, 64, 1, 4, 32, 2, 959, 943) \
    X(32, 128, 64, 1, 4, 32, 3, 563, 540) \
    X(32, 128, 128, 1, 4, 32, 2, 1065, 1035) \
    X(32, 64, 128, 1, 2, 32, 3, 636, 681)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 944, 1083) \
    X(16, 256, 128, 1, 4, 16, 2, 2269, 2220) \
    X(16, 128, 128, 1, 4, 16, 4, 1070, 1095) \
    X(16, 128, 256, 1, 4, 16, 2, 2524, 2428) \
    X(16, 64, 128, 1, 4, 16, 4, 467, 484) \
    X(16, 64, 256, 1, 4, 16, 3, 1335, 1430) \
    X(16, 32, 256, 1, 2, 16, 3, 835, 752) \
    X(16, 16, 256, 1, 1, 16, 3, 819, 737)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 2, 4, 16, 2, 3891, 3969) \
    X(256, 256, 64, 4, 2, 16, 2, 4044, 4101) \
    X(256, 128, 64, 2, 4, 16, 3, 2282, 2366) \
    X(128, 256, 64, 2, 4, 16, 3, 2259, 2347) \
    X(128, 128, 64, 2, 4, 16, 2, 1209, 1151) \
    X(128, 64, 64, 2, 4, 16, 3, 783, 750) \
    X(64, 128, 64, 2, 4, 16, 3, 769, 720) \
    X(128, 64, 64, 2, 4, 16, 2, 780, 804) \
    X(64, 128, 64, 2, 4, 16, 2, 791, 746) \
    X(64, 64, 64, 2, 4, 16, 3, 486, 461) \
    X(64, 64, 128, 2, 4, 16, 2, 938, 941) \
    X(128, 128, 64, 4, 2, 16, 2, 1216, 1149) \
    X(32, 64, 128, 1, 4, 16, 3, 635, 626)

// deeper LDS rings of tiles that win latency- and bandwidth-bound shapes (a request has NS-1 whole slabs
// of time to land); of eight such candidates these three were sweep-best on 10-20 % of the irregular shapes
#define G355_VARIANTS_BF16_5(X)    \
    X(64, 128, 64, 2, 4, 16, 4, 866, 901) \
    X(128, 128, 64, 2, 4, 16, 3, 1340, 1319) \
    X(128, 128, 64, 2, 4, 16, 4, 1332, 1323)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 4, 32, 2, 3779, 3834) \
    X(256, 256, 128, 2, 2, 32, 2, 4175, 4147) \
    X(256, 128, 128, 2, 4, 32, 3, 2287, 2318) \
    X(128, 256, 128, 2, 4, 32, 3, 2247, 2294) \
    X(128, 128, 128, 2, 2, 32, 2, 1089, 1113) \
    X(128, 128, 128, 2, 2, 32, 3, 1352, 1343) \
    X(128, 128, 256, 2, 2, 32, 2, 2835, 2856) \
    X(128, 64, 128, 2, 2, 32, 3, 829, 746) \
    X(64, 128, 128, 2, 2, 32, 3, 728, 737)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 1893, 1923) \
    X(64, 64, 128, 2, 2, 32, 3, 560, 504) \
    X(64, 64, 256, 2, 2, 32, 2, 1155, 1039) \
    X(64, 256, 128, 1, 4, 32, 2, 1195, 1205) \
    X(32, 256, 128, 1, 4, 32, 2, 964, 962) \
    X(32, 128, 256, 1, 4, 32, 2, 1109, 1107) \
    X(32, 32, 256, 1, 1, 32, 3, 793, 713) \
    X(16, 256, 256, 1, 4, 16, 2, 2614, 2492) \
    X(16, 128, 256, 1, 4, 16, 4, 1180, 1202) \
    X(16, 64, 256, 1, 4, 16, 4, 751, 676) \
    X(16, 16, 256, 1, 1, 16, 4, 671, 603)

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
