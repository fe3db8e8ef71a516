// Calibration probes (Section I of the paper: the model is parameterised by measurable
// hardware rates obtained with micro-benchmarks): the register-resident MFMA issue rate,
// which gives L_MI of Algorithm 3 and the achievable matrix-core ceiling, and the streaming
// read rate of HBM.  Both run synchronously on the given stream and time themselves with
// HIP events; they are not part of gemm_select or gemm_run.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm.h"

namespace {
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// 4 independent accumulator chains per wave, one wave per SIMD: enough to keep the pipe full.
template <int DT, int MI>
__global__ __launch_bounds__(256) void mfma_loop(float *out, int iters)
{
    f32x16 c[4] = {};
    f32x4 d[4] = {};
    bf16x8 a, b;
    for (int t = 0; t < 8; ++t) {
        a[t] = (__bf16)(float)(threadIdx.x & 3);
        b[t] = (__bf16)1.0f;
    }
    i32x8 ia, ib;
    for (int t = 0; t < 8; ++t) {
        ia[t] = 0x38383838;   // e4m3 1.0 in every byte
        ib[t] = 0x38383838;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (DT == GEMM_BF16 && MI == 32)
                c[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[q], 0, 0, 0);
            else if constexpr (DT == GEMM_BF16)
                d[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, d[q], 0, 0, 0);
            else if constexpr (MI == 32)
                c[q] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ia, ib, c[q], 0, 0, 0, 0, 0, 0);
            else
                d[q] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ia, ib, d[q], 0, 0, 0, 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int q = 0; q < 4; ++q) {
        for (int r = 0; r < 16; ++r)
            s += c[q][r];
        for (int r = 0; r < 4; ++r)
            s += d[q][r];
    }
    if (s == -1.0f)   // never true: keeps the loop alive
        out[0] = s;
}

__global__ __launch_bounds__(256) void stream_read(const uint4 *__restrict__ p, size_t n, uint32_t *out)
{
    uint4 acc = {0, 0, 0, 0};
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint4 v = p[i];
        acc.x ^= v.x;
        acc.y ^= v.y;
        acc.z ^= v.z;
        acc.w ^= v.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u)   // practically never
        out[0] = acc.x;
}

template <class F>
int timed(hipStream_t s, F &&launch, double *ms_out)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return GEMM_ERR_HIP;
    launch();   // warm-up
    (void)hipEventRecord(e0, s);
    launch();
    (void)hipEventRecord(e1, s);
    const hipError_t err = hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess || hipGetLastError() != hipSuccess)
        return GEMM_ERR_HIP;
    *ms_out = ms;
    return GEMM_OK;
}
}  // namespace

extern "C" int gemm_probe_mfma(int dtype, int mfma, void *scratch4, void *hip_stream, double *tflops_out)
{
    if (!scratch4 || !tflops_out)
        return GEMM_ERR_NULL;
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3)
        return GEMM_ERR_DTYPE;
    if (mfma != 32 && mfma != 16)
        return GEMM_ERR_CFG_ILLEGAL;
    hipStream_t s = (hipStream_t)hip_stream;
    const int iters = 20000, blocks = 1024;
    const double k = (dtype == GEMM_BF16) ? (mfma == 32 ? 16 : 32) : (mfma == 32 ? 64 : 128);
    const double flop = 2.0 * mfma * mfma * k * 4.0 /*chains*/ * iters * 4.0 /*waves*/ * blocks;
    double ms = 0;
    int rc;
    float *out = (float *)scratch4;
    (void)hipGetLastError();
    if (dtype == GEMM_BF16 && mfma == 32)
        rc = timed(s, [&] { hipLaunchKernelGGL((mfma_loop<GEMM_BF16, 32>), dim3(blocks), dim3(256), 0, s, out, iters); }, &ms);
    else if (dtype == GEMM_BF16)
        rc = timed(s, [&] { hipLaunchKernelGGL((mfma_loop<GEMM_BF16, 16>), dim3(blocks), dim3(256), 0, s, out, iters); }, &ms);
    else if (mfma == 32)
        rc = timed(s, [&] { hipLaunchKernelGGL((mfma_loop<GEMM_FP8_E4M3, 32>), dim3(blocks), dim3(256), 0, s, out, iters); }, &ms);
    else
        rc = timed(s, [&] { hipLaunchKernelGGL((mfma_loop<GEMM_FP8_E4M3, 16>), dim3(blocks), dim3(256), 0, s, out, iters); }, &ms);
    if (rc)
        return rc;
    *tflops_out = flop / (ms * 1e-3) * 1e-12;
    return GEMM_OK;
}

extern "C" int gemm_probe_stream(const void *buf, size_t bytes, void *scratch4, void *hip_stream, double *gbps_out)
{
    if (!buf || !scratch4 || !gbps_out)
        return GEMM_ERR_NULL;
    if (bytes < (size_t)1 << 20 || ((uintptr_t)buf & 15))
        return GEMM_ERR_ALIGN;
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t n = bytes / 16;
    double ms = 0;
    (void)hipGetLastError();
    const int rc = timed(
        s, [&] { hipLaunchKernelGGL(stream_read, dim3(2048), dim3(256), 0, s, (const uint4 *)buf, n, (uint32_t *)scratch4); },
        &ms);
    if (rc)
        return rc;
    *gbps_out = (double)(n * 16) / (ms * 1e-3) * 1e-9;
    return GEMM_OK;
}
