#pragma once
#include <hip/hip_runtime.h>

#include "gemm_kernel.hpp"

namespace g355 {
typedef hipError_t (*LaunchFn)(const KernelArgs &, hipStream_t);
LaunchFn kLaunchBf16_0(int), kLaunchBf16_1(int), kLaunchBf16_2(int), kLaunchBf16_3(int), kLaunchFp8_0(int), kLaunchFp8_1(int);
}  // namespace g355
