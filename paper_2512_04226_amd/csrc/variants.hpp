// The compiled kernel variants: the candidate tile list the selector ranks (Section V-B of
// the paper speaks of 75 searched configurations; Section V-E of 50-150 valid tiles per
// datatype).  One line per instantiation of gemm_kernel<>:
//   X(BLOCK_M, BLOCK_N, BLOCK_K, WAVES_M, WAVES_N, MFMA, LDS_STAGES, LOOP, LOOP_KC)
// LOOP / LOOP_KC: the K-loop form (0 to 6, see Tile in gemm_kernel.hpp) the instantiation for
// row-major / K-contiguous B is compiled with: the fastest of forms 0 to 4 on 8192^3 where one is
// at least 1.5 % faster than form 0 (bf16 and fp16 timings together for the 16-bit list), else 0;
// form 5 or 6 where it beat that choice by 3 % (form 6: 2 %) or more.
// The table holds no timing: the selector prices a variant from its shape and the hardware
// descriptor alone (Algorithm 3's instruction count times the measured issue interval, plus the
// slab's fill and synchronisation cost).
// The order is part of the ABI of kernel_id and of the selector's tie-break (earlier wins).
#pragma once

// bf16: BLOCK_K in elements; MFMA 32 -> v_mfma_f32_32x32x16_bf16, 16 -> v_mfma_f32_16x16x32_bf16
#define G355_VARIANTS_BF16_0(X)    \
    X(256, 256, 64, 2, 4, 32, 2, 3, 3) \
    X(256, 256, 64, 2, 2, 32, 2, 5, 4) \
    X(256, 256, 32, 2, 4, 32, 4, 3, 3) \
    X(256, 256, 32, 2, 2, 32, 4, 4, 4) \
    X(256, 256, 32, 2, 4, 32, 5, 3, 3) \
    X(256, 128, 64, 2, 4, 32, 3, 3, 5) \
    X(256, 128, 64, 2, 2, 32, 3, 5, 5) \
    X(128, 256, 64, 2, 4, 32, 3, 3, 1)
#define G355_VARIANTS_BF16_1(X)    \
    X(128, 256, 64, 2, 2, 32, 3, 5, 5) \
    X(128, 128, 64, 2, 2, 32, 2, 0, 0) \
    X(128, 128, 64, 2, 2, 32, 3, 5, 5) \
    X(64, 256, 64, 1, 4, 32, 2, 1, 0) \
    X(128, 64, 64, 2, 2, 32, 3, 5, 3) \
    X(64, 128, 64, 2, 2, 32, 3, 1, 3)
#define G355_VARIANTS_BF16_2(X)    \
    X(64, 64, 64, 2, 2, 32, 3, 3, 0) \
    X(64, 64, 128, 2, 2, 32, 2, 4, 0) \
    X(32, 256, 64, 1, 4, 32, 2, 2, 0) \
    X(32, 128, 64, 1, 4, 32, 3, 0, 0) \
    X(32, 128, 128, 1, 4, 32, 2, 0, 0) \
    X(32, 64, 128, 1, 2, 32, 3, 3, 1)
#define G355_VARIANTS_BF16_3(X)    \
    X(16, 256, 64, 1, 4, 16, 4, 5, 4) \
    X(16, 256, 128, 1, 4, 16, 2, 0, 3) \
    X(16, 128, 128, 1, 4, 16, 4, 3, 5) \
    X(16, 128, 256, 1, 4, 16, 2, 3, 3) \
    X(16, 64, 128, 1, 4, 16, 4, 0, 0) \
    X(16, 64, 256, 1, 4, 16, 3, 3, 1) \
    X(16, 32, 256, 1, 2, 16, 3, 0, 1) \
    X(16, 16, 256, 1, 1, 16, 3, 0, 2)
// 16x16x32 MFMA on the larger tiles, eight waves: fewer accumulator register bytes per flop than
// 32x32x16, which is what counts once the chip is power-limited.  The model prices the 4x2 and the 2x4 wave grid of
// the 256x256x64 tile alike; the 4x2 one measures 3-4 % faster on 8192^3 and is listed first (earlier wins a tie).
// On K-contiguous B the 2x4 grid in K-loop form 6 is the faster one (8192^3: 767 us against 794 bf16, 794 against 835
// fp16) and wins that tie there (variant_wins_tie_on_kc below).
// (A four-wave grid of this tile -- 128x128 wave tiles, accumulators in AGPRs, K-loop form 5 -- is level with the
// 4x2 grid on 8192^3 with row-major B and 3-4 % ahead with K-contiguous B, but 3-5 % behind on the irregular shapes
// that pick this tile: not listed.)
#define G355_VARIANTS_BF16_4(X)    \
    X(256, 256, 64, 4, 2, 16, 2, 4, 2) \
    X(256, 256, 64, 2, 4, 16, 2, 2, 6) \
    X(256, 128, 64, 2, 4, 16, 3, 3, 3) \
    X(128, 256, 64, 2, 4, 16, 3, 4, 3) \
    X(128, 128, 64, 2, 4, 16, 2, 2, 0) \
    X(64, 128, 64, 2, 4, 16, 3, 4, 1) \
    X(128, 64, 64, 2, 4, 16, 2, 0, 1) \
    X(64, 128, 64, 2, 4, 16, 2, 0, 0) \
    X(64, 64, 64, 2, 4, 16, 3, 0, 0) \
    X(64, 64, 128, 2, 4, 16, 2, 2, 0) \
    X(128, 128, 64, 4, 2, 16, 2, 1, 0) \
    X(32, 64, 128, 1, 4, 16, 3, 4, 3)

// deeper LDS rings of tiles that win latency- and bandwidth-bound shapes (a request has NS-1 whole slabs
// of time to land); of eight such candidates these three were sweep-best on 10-20 % of the irregular shapes
#define G355_VARIANTS_BF16_5(X)    \
    X(64, 128, 64, 2, 4, 16, 4, 2, 5) \
    X(128, 128, 64, 2, 4, 16, 3, 4, 1) \
    X(128, 128, 64, 2, 4, 16, 4, 3, 1)

// fp8 e4m3: MFMA 32 -> v_mfma_f32_32x32x64_f8f6f4, 16 -> v_mfma_f32_16x16x128_f8f6f4
#define G355_VARIANTS_FP8_0(X)     \
    X(256, 256, 128, 2, 2, 32, 2, 5, 5) \
    X(256, 256, 128, 2, 4, 32, 2, 2, 2) \
    X(256, 128, 128, 2, 4, 32, 3, 1, 5) \
    X(128, 256, 128, 2, 4, 32, 3, 4, 4) \
    X(128, 128, 128, 2, 2, 32, 2, 5, 5) \
    X(128, 128, 128, 2, 2, 32, 3, 5, 5) \
    X(128, 64, 128, 2, 2, 32, 3, 0, 4) \
    X(64, 128, 128, 2, 2, 32, 3, 0, 2)
#define G355_VARIANTS_FP8_1(X)     \
    X(64, 128, 256, 2, 2, 32, 3, 5, 5) \
    X(64, 64, 128, 2, 2, 32, 3, 0, 1) \
    X(64, 64, 256, 2, 2, 32, 2, 0, 3) \
    X(64, 256, 128, 1, 4, 32, 2, 0, 5) \
    X(32, 256, 128, 1, 4, 32, 2, 0, 0) \
    X(32, 128, 256, 1, 4, 32, 2, 0, 3) \
    X(32, 32, 256, 1, 1, 32, 3, 0, 4) \
    X(16, 256, 256, 1, 4, 16, 2, 1, 5) \
    X(16, 128, 256, 1, 4, 16, 4, 5, 3) \
    X(16, 64, 256, 1, 4, 16, 4, 0, 5) \
    X(16, 16, 256, 1, 1, 16, 4, 0, 4)

#define G355_VARIANTS_BF16(X) \
    G355_VARIANTS_BF16_0(X) G355_VARIANTS_BF16_1(X) G355_VARIANTS_BF16_2(X) G355_VARIANTS_BF16_3(X) G355_VARIANTS_BF16_4(X) \
    G355_VARIANTS_BF16_5(X)
#define G355_VARIANTS_FP8(X) G355_VARIANTS_FP8_0(X) G355_VARIANTS_FP8_1(X)

namespace g355 {
struct Variant {
    int block_m, block_n, block_k, waves_m, waves_n, mfma, stages;
};
// Ties between equal predictions go to the earlier entry of the list, with one exception per B layout that the
// lists' single order cannot express: on K-contiguous B the 2x4 wave grid of the 16-bit 256x256x64 tile with the
// 16x16x32 MFMA goes before the 4x2 grid it ties with.
inline bool variant_wins_tie_on_kc(const Variant &v)
{
    return v.block_m == 256 && v.block_n == 256 && v.block_k == 64 && v.waves_m == 2 && v.waves_n == 4 && v.mfma == 16 &&
           v.stages == 2;
}
// Spatial K-unroll factors offered with every variant.
constexpr int kSplitKs[] = {1, 2, 4, 8, 16, 32};
constexpr int kNumSplitKs = sizeof(kSplitKs) / sizeof(kSplitKs[0]);
// Work splits offered with every variant: the split-K factors, then stream-K.
constexpr int kNumSplits = kNumSplitKs + 1;
inline int split_k_of(int mode) { return mode < kNumSplitKs ? kSplitKs[mode] : 1; }
inline int stream_k_of(int mode) { return mode == kNumSplitKs ? 1 : 0; }
}  // namespace g355
