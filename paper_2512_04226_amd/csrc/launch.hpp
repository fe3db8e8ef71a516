#pragma once
#include <hip/hip_runtime.h>

#include "gemm_kernel.hpp"

namespace g355 {
typedef hipError_t (*LaunchFn)(const KernelArgs &, hipStream_t);
typedef hipError_t (*OccupancyFn)(int *blocks_per_cu);
struct VariantFns {
    LaunchFn launch;
    OccupancyFn occupancy;   // the runtime's resident-workgroups-per-CU figure for the instantiation
};
// (variant index inside the translation unit's list, storage of B: 0 row-major K x N, 1 K-contiguous N x K,
//  1 for the instantiation that handles an N or K that is not a whole number of 16-byte chunks)
const VariantFns &kLaunchBf16_0(int, int, int),
    &kLaunchBf16_1(int, int, int),
    &kLaunchBf16_2(int, int, int),
    &kLaunchBf16_3(int, int, int),
    &kLaunchFp8_0(int, int, int),
    &kLaunchFp8_1(int, int, int),
    &kLaunchFp16_0(int, int, int),
    &kLaunchFp16_1(int, int, int),
    &kLaunchFp16_2(int, int, int),
    &kLaunchFp16_3(int, int, int),
    &kLaunchBf16_4(int, int, int),
    &kLaunchFp16_4(int, int, int),
    &kLaunchBf16_5(int, int, int),
    &kLaunchFp16_5(int, int, int);   // fp16 shares the bf16 variant lists
}  // namespace g355
