// Calibration probes (Section I of the paper: the model is parameterised by measurable
// hardware rates obtained with micro-benchmarks).  One probe per entry of the hardware
// descriptor H that the device itself can report:
//   gemm_probe_mfma / _ex   register-resident MFMA loop  -> L_MI of Algorithm 3 and the matrix-core
//                           ceiling, on constant operands or on operands drawn like the workloads'
//   gemm_probe_stream       one streaming read of a buffer -> R_MEM (HBM) of Algorithm 7
//   gemm_probe_read         repeated reads of a buffer whose size decides which level serves them
//                           -> R_1 (L2), R_2 (MALL), R_MEM
//   gemm_probe_lds          LDS fragment-read loops -> the LDS term's rates (plain and transpose reads)
//   gemm_probe_fill         64 KB slabs moved from global memory into LDS by 8-wave workgroups -> the
//                           per-CU rate of the kernel's refill path
//   gemm_probe_latency      dependent loads through a buffer -> L_lat of Algorithm 7
// All run synchronously on the given stream and time themselves with HIP events; none is part
// of gemm_select or gemm_run.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gemm.h"

namespace {
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

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


// ---- MFMA loop on workload-like operands ----
// A wave holds TM column fragments and TN row fragments in two register sets and alternates
// between them, as the GEMM kernel's double-buffered k-steps do, accumulating TM x TN tiles:
// the matrix cores see different operand bits in every instruction and the accumulators wander
// like real partial sums.  RND = 0 fills the same registers with constants (lane & 3, 1.0).
__device__ inline uint32_t probe_hash(uint32_t x)
{
    // an integer mixer (xor-shift and odd multiplications); only the spread of the bits matters here
    x ^= x >> 17;
    x *= 0xed5ad4bbu;
    x ^= x >> 11;
    x *= 0xac4c1b51u;
    x ^= x >> 15;
    x *= 0x31848babu;
    x ^= x >> 14;
    return x;
}
__device__ inline float probe_normal(uint32_t &ctr)
{
    // Box-Muller on two hashed uniforms in (0, 1]
    const float u1 = (float)((probe_hash(ctr++) >> 8) + 1) * (1.0f / 16777216.0f);
    const float u2 = (float)(probe_hash(ctr++) >> 8) * (1.0f / 16777216.0f);
    return __builtin_sqrtf(-2.0f * __builtin_logf(u1)) * __builtin_cosf(6.2831853f * u2);
}
// fp32 -> e4m3 (OCP: bias 7, 3 mantissa bits, max 448, no infinity), round to nearest even, saturating
__device__ inline uint32_t probe_e4m3(float x)
{
    const uint32_t sign = x < 0.f ? 0x80u : 0u;
    float a = __builtin_fabsf(x);
    if (!(a < 448.f))
        return sign | 0x7eu;
    if (a < 0.015625f) {   // subnormals: multiples of 2^-9
        return sign | (uint32_t)__builtin_rintf(a * 512.f);
    }
    int e;
    const float m = __builtin_frexpf(a, &e);              // a = m * 2^e, m in [0.5, 1)
    uint32_t q = (uint32_t)__builtin_rintf(m * 16.f);     // 8 .. 16
    int be = e - 1 + 7;
    if (q == 16) {
        q = 8;
        ++be;
    }
    return sign | ((uint32_t)be << 3) | (q - 8);
}

template <int DT, int MI, int RND>
__global__ __launch_bounds__(256) void mfma_tile_loop(float *out, int iters, uint32_t seed)
{
    constexpr int TM = (MI == 32) ? 2 : 4, TN = 4;
    constexpr int REGS = (DT == GEMM_BF16) ? 4 : 8;        // operand registers per fragment
    typedef float acc_t __attribute__((ext_vector_type(MI == 32 ? 16 : 4)));
    typedef int frag_t __attribute__((ext_vector_type(REGS)));
    frag_t a[2][TM], b[2][TN];
    uint32_t ctr = probe_hash(seed + blockIdx.x * 256u + threadIdx.x) | 1u;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int f = 0; f < TM + TN; ++f) {
            frag_t v;
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                uint32_t w;
                if constexpr (RND == 0) {
                    w = (DT == GEMM_BF16) ? 0x3f803f80u : 0x38383838u;   // 1.0 in every element
                } else if constexpr (DT == GEMM_BF16) {
                    const uint32_t lo = __builtin_bit_cast(uint32_t, probe_normal(ctr)) + 0x8000u;
                    const uint32_t hi = __builtin_bit_cast(uint32_t, probe_normal(ctr)) + 0x8000u;
                    w = (lo >> 16) | (hi & 0xffff0000u);
                } else {
                    // N(0,1) scaled so that the largest of ~1e8 draws lands on 448, as config 4 scales its tensors
                    w = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        w |= probe_e4m3(probe_normal(ctr) * (448.f / 5.6f)) << (8 * q);
                }
                v[r] = (int)w;
            }
            if (f < TM)
                a[s][f] = v;
            else
                b[s][f - TM] = v;
        }
    acc_t acc[TN][TM];
    for (int j = 0; j < TN; ++j)
        for (int i = 0; i < TM; ++i)
            for (int r = 0; r < (MI == 32 ? 16 : 4); ++r)
                acc[j][i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if constexpr (DT == GEMM_BF16 && MI == 32)
                        acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b[s][j]),
                                                                            __builtin_bit_cast(bf16x8, a[s][i]), acc[j][i], 0, 0, 0);
                    else if constexpr (DT == GEMM_BF16)
                        // written out, with the accumulator tied to one vector register quad: left to the
                        // register allocator this loop moves every accumulator through the accumulation
                        // registers between its two updates (three extra vector instructions per MFMA).
                        // An accumulator is next touched 16 instructions later: no wait states are needed.
                        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[j][i]) : "v"(b[s][j]), "v"(a[s][i]));
                    else if constexpr (MI == 32)
                        acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[s][j], a[s][i], acc[j][i], 0, 0, 0, 0, 0, 0);
                    else
                        acc[j][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[s][j], a[s][i], acc[j][i], 0, 0, 0, 0, 0, 0);
                }
    }
    // the last written-out MFMAs have left the pipeline before their results are read
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float sum = 0.f;
    for (int j = 0; j < TN; ++j)
        for (int i = 0; i < TM; ++i)
            for (int r = 0; r < (MI == 32 ? 16 : 4); ++r)
                sum += acc[j][i][r];
    if (sum == -1.2345e-30f)   // practically never: keeps the loop alive
        out[0] = sum;
}

// ---- repeated reads: every workgroup re-reads its own grid-strided share of the buffer `passes` times ----
__global__ __launch_bounds__(256) void read_passes(const uint4 *__restrict__ p, size_t n, int passes, uint32_t *out)
{
    uint4 acc = {0, 0, 0, 0};
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (int pass = 0; pass < passes; ++pass) {
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
            const uint4 v = p[i];
            acc.x ^= v.x;
            acc.y ^= v.y;
            acc.z ^= v.z;
            acc.w ^= v.w;
        }
        // the next pass must load again: the compiler may not keep values across this point
        asm volatile("" ::: "memory");
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u)   // practically never
        out[0] = acc.x;
}

// ---- LDS fragment reads: KIND 0 ds_read_b128, 1 ds_read_b64, 2 ds_read_b64_tr_b16, 3 ds_read_b64_tr_b8 ----
// Linear, conflict-free addresses (lane * width); eight reads in flight per wave.
#define PROBE_LDS __attribute__((address_space(3)))
typedef int i32x4p __attribute__((ext_vector_type(4)));
typedef int i32x2p __attribute__((ext_vector_type(2)));
typedef short s16x4p __attribute__((ext_vector_type(4)));
template <int KIND>
__global__ __launch_bounds__(512) void lds_read_loop(uint32_t *out, int iters)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[64 * 1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 64 * 1024 / 4; i += blockDim.x)
        ((PROBE_LDS uint32_t *)smem)[i] = (uint32_t)i;
    __syncthreads();
    constexpr int W = (KIND == 0) ? 16 : 8;                       // bytes per lane and read
    PROBE_LDS uint8_t *base = (PROBE_LDS uint8_t *)smem + (wave & 7) * 8192 + lane * W;
    int acc = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            PROBE_LDS uint8_t *q = base + u * (64 * W);           // 8 x 1 KB or 8 x 512 B, inside the wave's 8 KB
            if constexpr (KIND == 0) {
                i32x4p v;
                asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"((uint32_t)(uintptr_t)q) : "memory");
                asm volatile("s_waitcnt lgkmcnt(7)" ::: "memory");
                acc += v[0];
            } else if constexpr (KIND == 1) {
                i32x2p v;
                asm volatile("ds_read_b64 %0, %1" : "=v"(v) : "v"((uint32_t)(uintptr_t)q) : "memory");
                asm volatile("s_waitcnt lgkmcnt(7)" ::: "memory");
                acc += v[0];
            } else if constexpr (KIND == 2) {
                const s16x4p v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((PROBE_LDS s16x4p *)q);
                acc += v[0];
            } else {
                const i32x2p v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((PROBE_LDS i32x2p *)q);
                acc += v[0];
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (acc == 0x12345677)   // practically never
        out[0] = (uint32_t)acc;
}

// ---- slab fill: workgroups of 8 waves move 64 KB "slabs" from global memory towards LDS ----
// Every wave issues the requests of 8 of a slab's 64 one-KB units (16 bytes per lane), as the GEMM
// kernel's refill does, with at most two slabs' requests in flight.
//   KIND 0  buffer loads that write LDS directly, 16 bytes per lane
//   KIND 1  the same path 4 bytes per lane (four times the instructions)
//   KIND 2  buffer loads into registers (the data goes nowhere)
//   KIND 3  buffer loads into registers, then ds_write_b128 into the lane's LDS slot
//   PAT 0   a slab is 64 KB of consecutive bytes; workgroups start 17 slabs apart inside the window
//   PAT 1   a slab is 512 rows of 128 bytes, rows 16 KB apart (a K slab of a row-major bf16 operand
//           with K = 8192); successive slabs step 128 bytes along the rows inside `span` bytes
//   PAT 2/3 a slab is 512 pieces of 128 bytes / 128 pieces of 512 bytes of consecutive rows 16 KB apart;
//           successive slabs take the next block of rows of the window, then the next piece of the rows:
//           every byte of the window is read once before any is read again
typedef unsigned u32x4p __attribute__((ext_vector_type(4)));
template <int KIND, int PAT>
__global__ __launch_bounds__(512) void fill_loop(const uint8_t *buf, unsigned window, unsigned span, int iters, int sync,
                                                 uint32_t *out)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[64 * 1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(buf), 0, window, 0x00020000);
    PROBE_LDS uint8_t *lds = (PROBE_LDS uint8_t *)smem;
    // byte offset of this lane's 16 bytes of unit u in slab `it`; always below `window`
    auto offset_of = [&](int it, int u, int sub) -> unsigned {
        const unsigned unit = (unsigned)(u * 8 + wave);
        if constexpr (PAT == 0) {
            const unsigned base = ((blockIdx.x * 17u + (unsigned)it) * 65536u + unit * 1024u) & (window - 1);
            return KIND == 1 ? base + sub * 256u + lane * 4u : base + lane * 16u;
        } else if constexpr (PAT == 1) {
            const unsigned kofs = ((unsigned)it * 128u) & (span - 1);
            if constexpr (KIND == 1)
                return (unit * 8u + sub * 2u + (lane >> 5)) * 16384u + kofs + (lane & 31) * 4u;
            return (unit * 8u + (lane >> 3)) * 16384u + kofs + (lane & 7) * 16u;
        } else {
            // slab j of the launch: block of 65536 / PIECE rows j mod (row blocks), piece (j / row blocks) of the rows
            constexpr unsigned PIECE = PAT == 2 ? 128u : 512u, ROWS = 65536u / PIECE, LPP = PIECE / 16u;
            const unsigned j = blockIdx.x * 17u + (unsigned)it, blocks = (window >> 14) / ROWS;
            const unsigned rb = j % blocks, kofs = ((j / blocks) * PIECE) & 16383u;
            return (rb * ROWS + unit * (64u / LPP) + lane / LPP) * 16384u + kofs + (lane % LPP) * 16u;
        }
    };
    if constexpr (KIND <= 1) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if constexpr (KIND == 0) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass does not know the 16-byte form and drops the launch stub
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (PROBE_LDS void *)(lds + (u * 8 + wave) * 1024), 16,
                                                             offset_of(it, u, 0), 0, 0, 0);
#endif
                } else {
#pragma unroll
                    for (int sub = 0; sub < 4; ++sub)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (PROBE_LDS void *)(lds + (u * 8 + wave) * 1024 + sub * 256), 4,
                                                                 offset_of(it, u, sub), 0, 0, 0);
                }
            }
            if constexpr (KIND == 0)
                asm volatile("s_waitcnt vmcnt(8)" ::: "memory");     // the previous slab has landed
            else
                asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
            if (sync)
                __builtin_amdgcn_s_barrier();   // the bare barrier: outstanding loads stay in flight across it
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        u32x4p cur[8], nxt[8];
        unsigned acc = 0;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            cur[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, offset_of(0, u, 0), 0, 0);
        for (int it = 1; it <= iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                nxt[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, offset_of(it < iters ? it : 0, u, 0), 0, 0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if constexpr (KIND == 2)
                    asm volatile("" ::"v"(cur[u]));
                else
                    *(PROBE_LDS u32x4p *)(lds + (u * 8 + wave) * 1024 + lane * 16) = cur[u];
                cur[u] = nxt[u];
            }
            if (sync)
                __builtin_amdgcn_s_barrier();   // the bare barrier: outstanding loads stay in flight across it
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc ^= cur[u][0];
        if (acc == 0x9E3779B9u && out)   // practically never
            out[1] = acc;
    }
    __syncthreads();
    if (((PROBE_LDS uint32_t *)smem)[tid] == 0x9E3779B9u && iters < 0)   // never: keeps the LDS writes alive
        out[0] = 1;
}

// ---- dependent loads: one lane follows a chain of line indices through the buffer ----
// Line i (128 bytes apart) of the first `chain` lines holds the index of line (i + step) mod chain; step is
// odd and chain a power of two, so the chain visits every one of them before it repeats.  All `lines` lines
// of the buffer are written, in ascending order: what the caches still hold afterwards is the END of the
// buffer, so a chain confined to the first half starts from the level the buffer's size selects.
__global__ void chase_init(uint32_t *p, uint32_t lines, uint32_t chain, uint32_t step)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < lines; i += gridDim.x * blockDim.x)
        p[(size_t)i * 32] = (i + step) & (chain - 1);
}
__global__ void chase_loop(const uint32_t *p, uint32_t chain, uint32_t start, int hops, uint32_t *out)
{
    if (threadIdx.x != 0 || blockIdx.x != 0)
        return;
    uint32_t j = start;
    for (int h = 0; h < hops; ++h)
        j = *(const volatile uint32_t *)(p + (size_t)(j & (chain - 1)) * 32);   // the mask keeps any value in range
    out[0] = j;
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


// Launch `launch` untimed for about warm_ms, then timed for about timed_ms (at least twice each):
// after an idle gap the chip boosts, then throttles, and settles only after 15-20 ms of work.
template <class F>
static int timed_settled(hipStream_t s, F &&launch, double warm_ms, double timed_ms, double *ms_per_launch)
{
    double one = 0;
    int rc = timed(s, launch, &one);
    if (rc)
        return rc;
    if (!(one > 1e-4))
        one = 1e-4;
    int n_warm = (int)(warm_ms / one) + 1, n_timed = (int)(timed_ms / one) + 1;
    n_warm = n_warm > 2000 ? 2000 : n_warm;
    n_timed = n_timed > 2000 ? 2000 : (n_timed < 2 ? 2 : n_timed);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return GEMM_ERR_HIP;
    for (int i = 0; i < n_warm; ++i)
        launch();
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < n_timed; ++i)
        launch();
    (void)hipEventRecord(e1, s);
    const hipError_t err = hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess || hipGetLastError() != hipSuccess)
        return GEMM_ERR_HIP;
    *ms_per_launch = ms / n_timed;
    return GEMM_OK;
}

extern "C" int gemm_probe_mfma_ex(int dtype, int mfma, int operands, double warm_ms, double timed_ms, void *scratch4,
                                  void *hip_stream, double *tflops_out)
{
    if (!scratch4 || !tflops_out)
        return GEMM_ERR_NULL;
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3)
        return GEMM_ERR_DTYPE;
    if ((mfma != 32 && mfma != 16) || (operands != 0 && operands != 1) || !(warm_ms >= 0) || !(timed_ms > 0) ||
        warm_ms > 1000 || timed_ms > 1000)
        return GEMM_ERR_CFG_ILLEGAL;
    hipStream_t s = (hipStream_t)hip_stream;
    const int iters = 2000, blocks = 1024;
    const double k = (dtype == GEMM_BF16) ? (mfma == 32 ? 16 : 32) : (mfma == 32 ? 64 : 128);
    const double per_iter = 2.0 /*sets*/ * 4 /*TN*/ * (mfma == 32 ? 2 : 4) /*TM*/;
    const double flop = 2.0 * mfma * mfma * k * per_iter * iters * 4.0 /*waves*/ * blocks;
    float *out = (float *)scratch4;
    double ms = 0;
    int rc;
    (void)hipGetLastError();
#define PROBE_GO(DT, MI, R)                                                                                              \
    rc = timed_settled(                                                                                                  \
        s, [&] { hipLaunchKernelGGL((mfma_tile_loop<DT, MI, R>), dim3(blocks), dim3(256), 0, s, out, iters, 12345u); }, \
        warm_ms, timed_ms, &ms)
    if (dtype == GEMM_BF16 && mfma == 32 && operands)
        PROBE_GO(GEMM_BF16, 32, 1);
    else if (dtype == GEMM_BF16 && mfma == 32)
        PROBE_GO(GEMM_BF16, 32, 0);
    else if (dtype == GEMM_BF16 && operands)
        PROBE_GO(GEMM_BF16, 16, 1);
    else if (dtype == GEMM_BF16)
        PROBE_GO(GEMM_BF16, 16, 0);
    else if (mfma == 32 && operands)
        PROBE_GO(GEMM_FP8_E4M3, 32, 1);
    else if (mfma == 32)
        PROBE_GO(GEMM_FP8_E4M3, 32, 0);
    else if (operands)
        PROBE_GO(GEMM_FP8_E4M3, 16, 1);
    else
        PROBE_GO(GEMM_FP8_E4M3, 16, 0);
#undef PROBE_GO
    if (rc)
        return rc;
    *tflops_out = flop / (ms * 1e-3) * 1e-12;
    return GEMM_OK;
}

extern "C" int gemm_probe_mfma(int dtype, int mfma, void *scratch4, void *hip_stream, double *tflops_out)
{
    // constant operands, 10 ms of untimed launches before 10 ms of timed ones
    return gemm_probe_mfma_ex(dtype, mfma, 0, 10.0, 10.0, scratch4, hip_stream, tflops_out);
}

extern "C" int gemm_probe_read(const void *buf, size_t bytes, int passes, void *scratch4, void *hip_stream, double *gbps_out)
{
    if (!buf || !scratch4 || !gbps_out)
        return GEMM_ERR_NULL;
    if (bytes < (size_t)1 << 20 || ((uintptr_t)buf & 15))
        return GEMM_ERR_ALIGN;
    if (passes < 1 || passes > 4096)
        return GEMM_ERR_SHAPE;
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t n = bytes / 16;
    double ms = 0;
    (void)hipGetLastError();
    const int rc = timed(
        s, [&] { hipLaunchKernelGGL(read_passes, dim3(2048), dim3(256), 0, s, (const uint4 *)buf, n, passes, (uint32_t *)scratch4); },
        &ms);
    if (rc)
        return rc;
    *gbps_out = (double)(n * 16) * passes / (ms * 1e-3) * 1e-9;
    return GEMM_OK;
}

extern "C" int gemm_probe_lds(int kind, int waves_per_cu, void *scratch4, void *hip_stream, double *gbps_out)
{
    if (!scratch4 || !gbps_out)
        return GEMM_ERR_NULL;
    if (kind < 0 || kind > 3 || (waves_per_cu != 4 && waves_per_cu != 8 && waves_per_cu != 16))
        return GEMM_ERR_CFG_ILLEGAL;
    hipStream_t s = (hipStream_t)hip_stream;
    // one workgroup of 4 or 8 waves per CU (64 KB of LDS each; two of 8 waves for 16 per CU), two rounds
    const int threads = waves_per_cu == 4 ? 256 : 512;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus < 1) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    const int blocks = cus * (waves_per_cu == 16 ? 2 : 1) * 2;
    const int iters = 4000;
    const double bytes = (double)blocks * (threads / 64) * iters * 8.0 * 64.0 * (kind == 0 ? 16 : 8);
    uint32_t *out = (uint32_t *)scratch4;
    double ms = 0;
    int rc;
    (void)hipGetLastError();
    if (kind == 0)
        rc = timed(s, [&] { hipLaunchKernelGGL(lds_read_loop<0>, dim3(blocks), dim3(threads), 0, s, out, iters); }, &ms);
    else if (kind == 1)
        rc = timed(s, [&] { hipLaunchKernelGGL(lds_read_loop<1>, dim3(blocks), dim3(threads), 0, s, out, iters); }, &ms);
    else if (kind == 2)
        rc = timed(s, [&] { hipLaunchKernelGGL(lds_read_loop<2>, dim3(blocks), dim3(threads), 0, s, out, iters); }, &ms);
    else
        rc = timed(s, [&] { hipLaunchKernelGGL(lds_read_loop<3>, dim3(blocks), dim3(threads), 0, s, out, iters); }, &ms);
    if (rc)
        return rc;
    *gbps_out = bytes / (ms * 1e-3) * 1e-9;
    return GEMM_OK;
}

extern "C" int gemm_probe_fill(int kind, int pattern, int wgs_per_cu, int sync, const void *buf, size_t bytes,
                               size_t footprint, void *scratch4, void *hip_stream, double *gbps_out)
{
    if (!buf || !scratch4 || !gbps_out)
        return GEMM_ERR_NULL;
    if (kind < 0 || kind > 3 || pattern < 0 || pattern > 3 || wgs_per_cu < 1 || wgs_per_cu > 2 || (pattern >= 2 && kind == 1))
        return GEMM_ERR_CFG_ILLEGAL;
    if ((uintptr_t)buf & 127)
        return GEMM_ERR_ALIGN;
    // patterns 0, 2, 3: the window is `footprint` bytes (a power of two, 64 KiB (8 MiB) .. 2 GiB); pattern 1: 512 rows 16 KiB
    // apart (an 8 MiB window) of which the first `footprint` bytes (128 .. 16384, a power of two) are read
    unsigned window, span = 128;
    if (footprint & (footprint - 1))
        return GEMM_ERR_ALIGN;
    if (pattern == 0 || pattern >= 2) {
        if (footprint < (pattern ? (size_t)8 << 20 : 65536) || footprint > ((size_t)1 << 31) || footprint > bytes)
            return GEMM_ERR_ALIGN;
        window = (unsigned)footprint;
    } else {
        if (footprint < 128 || footprint > 16384 || bytes < ((size_t)8 << 20))
            return GEMM_ERR_ALIGN;
        window = 8u << 20;
        span = (unsigned)footprint;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus < 1) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    const int blocks = cus * wgs_per_cu, iters = 2048 / wgs_per_cu;
    const double moved = (double)blocks * iters * 65536.0;
    const uint8_t *p = (const uint8_t *)buf;
    uint32_t *out = (uint32_t *)scratch4;
    double ms = 0;
    (void)hipGetLastError();
#define FILL_CASE(K, P)                                                                                                       \
    if (kind == K && pattern == P)                                                                                            \
        rc = timed(s, [&] { hipLaunchKernelGGL((fill_loop<K, P>), dim3(blocks), dim3(512), 0, s, p, window, span, iters, sync, out); }, &ms);
    int rc = GEMM_ERR_CFG_ILLEGAL;
    FILL_CASE(0, 0) FILL_CASE(1, 0) FILL_CASE(2, 0) FILL_CASE(3, 0) FILL_CASE(0, 1) FILL_CASE(1, 1) FILL_CASE(2, 1) FILL_CASE(3, 1)
    FILL_CASE(0, 2) FILL_CASE(2, 2) FILL_CASE(3, 2) FILL_CASE(0, 3) FILL_CASE(2, 3) FILL_CASE(3, 3)
#undef FILL_CASE
    if (rc)
        return rc;
    *gbps_out = moved / (ms * 1e-3) * 1e-9;
    return GEMM_OK;
}

extern "C" int gemm_probe_latency(void *buf, size_t bytes, void *scratch4, void *hip_stream, double *ns_out)
{
    if (!buf || !scratch4 || !ns_out)
        return GEMM_ERR_NULL;
    if (bytes < (size_t)1 << 20 || ((uintptr_t)buf & 127))
        return GEMM_ERR_ALIGN;
    // the largest power-of-two number of 128-byte lines that fits (at most 2^25 lines = 4 GiB)
    uint32_t lines = 1;
    while ((size_t)lines * 2 * 128 <= bytes && lines < (1u << 25))
        lines *= 2;
    hipStream_t s = (hipStream_t)hip_stream;
    const int hops = 4096;
    // Small buffers (an L2's worth): the chain covers the whole buffer and the timed walk repeats the
    // warm-up walk's lines, which that walk left in the L2 of the XCD the single workgroup runs on.
    // Larger ones: the chain lives in the first half and the timed walk continues where the warm-up
    // walk stopped, on lines that no walk has touched since they were written.
    const bool l2_level = bytes <= ((size_t)4 << 20);
    const uint32_t chain = l2_level ? lines : lines / 2;
    // an odd step of an eighth of the chain plus a bit: consecutive hops land in different channels and pages
    const uint32_t step = (chain / 8 + 1237u) | 1u;
    (void)hipGetLastError();
    hipLaunchKernelGGL(chase_init, dim3(1024), dim3(256), 0, s, (uint32_t *)buf, lines, chain, step);
    if (hipGetLastError() != hipSuccess)
        return GEMM_ERR_HIP;
    double ms = 0, ms0 = 0;
    // the launch's own fixed cost is measured with a zero-hop run and taken off
    int rc = timed(s, [&] { hipLaunchKernelGGL(chase_loop, dim3(1), dim3(64), 0, s, (const uint32_t *)buf, chain, 0u, 0, (uint32_t *)scratch4); }, &ms0);
    if (rc)
        return rc;
    int call = 0;
    rc = timed(
        s,
        [&] {
            const uint32_t start = l2_level ? 0u : (uint32_t)(((uint64_t)call * hops * step) & (chain - 1));
            ++call;
            hipLaunchKernelGGL(chase_loop, dim3(1), dim3(64), 0, s, (const uint32_t *)buf, chain, start, hops, (uint32_t *)scratch4);
        },
        &ms);
    if (rc)
        return rc;
    *ns_out = (ms - ms0) * 1e6 / hops;
    return GEMM_OK;
}
