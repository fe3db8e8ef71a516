// gemm_run and the split-K workspace: the only entry points that touch the GPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstddef>
#include <cstring>
#include <mutex>

#include "../../include/gemm.h"
#include "gemm_kernel.hpp"
#include "launch.hpp"
#include "model.hpp"

using namespace g355;

namespace g355 {
// Sum the split-K slabs in slice order (deterministic), scale, round to bf16.
// Scale four sums, add beta * C when beta != 0 (C is read before it is overwritten), round to
// the 16-bit output format (f16 != 0: IEEE fp16, else bf16) and store.
__device__ inline void scale_round_store(f32x4 s, float alpha, float beta, void *dst, int f16, int count = 4)
{
    // count < 4: the ragged right edge of C -- only the first `count` outputs exist; C is read (beta != 0)
    // as a whole quad all the same, which stays inside the row's leading dimension
    if (f16) {
        f16x4 o;
        const f16x4 c = (beta != 0.f) ? *(const f16x4 *)dst : f16x4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r)
            o[r] = (beta != 0.f) ? (_Float16)__builtin_fmaf(beta, (float)c[r], s[r] * alpha) : (_Float16)(s[r] * alpha);
        if (count >= 4) {
            *(f16x4 *)dst = o;
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r)
                if (r < count)
                    ((_Float16 *)dst)[r] = o[r];
        }
    } else {
        bf16x4 o;
        const bf16x4 c = (beta != 0.f) ? *(const bf16x4 *)dst : bf16x4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r)
            o[r] = (beta != 0.f) ? (__bf16)__builtin_fmaf(beta, (float)c[r], s[r] * alpha) : (__bf16)(s[r] * alpha);
        if (count >= 4) {
            *(bf16x4 *)dst = o;
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r)
                if (r < count)
                    ((__bf16 *)dst)[r] = o[r];
        }
    }
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ ws, uint16_t *C, int M, int N, int ldc,
                                                            int split_k, float alpha, float beta, int f16,
                                                            long long stride_c)
{
    // slab rows are N rounded up to 8 floats apart (the kernels store whole 32-byte pieces also at a ragged edge)
    const size_t nw = (size_t)(N + 7) / 8 * 8;
    ws += (size_t)blockIdx.y * split_k * M * nw;     // problem of the batch
    C += (size_t)blockIdx.y * stride_c;
    const size_t qpr = (size_t)(N + 3) / 4;          // quads per row, the last one possibly partial
    const size_t quads = (size_t)M * qpr;
    const size_t slab = (size_t)M * nw;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += (size_t)gridDim.x * blockDim.x) {
        const size_t m = q / qpr, n = (q % qpr) * 4;
        const float *p = ws + m * nw + n;
        f32x4 s = *(const f32x4 *)p;
        for (int k = 1; k < split_k; ++k) {
            f32x4 t = *(const f32x4 *)(p + k * slab);
            s += t;
        }
        const int count = (int)((size_t)N - n < 4 ? (size_t)N - n : 4);
        scale_round_store(s, alpha, beta, C + m * ldc + n, f16, count);
    }
}


// Stream-K second pass: for every stream-K tile that more than one worker contributed to,
// sum the workers' fp32 partial tiles, scale, round to bf16.  A block of 256 threads is R
// thread rows of 256 / R groups of 4 consecutive outputs; the rows share the contributor
// list (row r adds contributors r, r + R, ... in worker order) and are combined through LDS
// as a fixed binary tree.  The host picks R from the number of contributors per tile, so
// the result depends only on the plan: deterministic.
template <int R>
__global__ __launch_bounds__(256) void streamk_sum_kernel(const float *__restrict__ ws, uint16_t *C, int M, int N, int ldc,
                                                          float alpha, float beta, int f16, int tiles_m, int tiles_n,
                                                          int group_m, SkPlan sk, int BM, int BN, int blocks_per_tile)
{
    constexpr int Q = 256 / R;
    __shared__ f32x4 part[R][Q];
    const int j = blockIdx.x / blocks_per_tile;
    const int quad = threadIdx.x % Q, r = threadIdx.x / Q;
    const int q = (blockIdx.x % blocks_per_tile) * Q + quad;
    int g_first, g_last;
    sk_contributors(sk, j, &g_first, &g_last);
    if (g_first == g_last)
        return;   // one worker computed the whole tile and stored it (uniform over the block)
    int tm, tn;
    logical_tile(tiles_m, tiles_n, group_m, sk.dp_tiles + j, tm, tn);
    const int row = q / (BN / 4), col = (q % (BN / 4)) * 4;
    const int m = tm * BM + row, n = tn * BN + col;
    const bool live = q < BM * BN / 4 && m < M && n < N;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        const size_t tile_elems = (size_t)BM * BN;
        const float *base = ws + (size_t)row * BN + col;
        // the first contributor's partial is its second segment unless its range starts with
        // this tile; every later contributor's range starts inside this tile (first segment)
        const int slot_first = sk_slot_of(sk, g_first, j);
#pragma unroll 4
        for (int g = g_first + r; g <= g_last; g += R) {
            const int slot = (g == g_first) ? slot_first : 0;
            s += *(const f32x4 *)(base + (size_t)(2 * g + slot) * tile_elems);
        }
    }
    if constexpr (R > 1) {
        part[r][quad] = s;
        __syncthreads();
#pragma unroll
        for (int half = R / 2; half >= 1; half /= 2) {
            if (r < half)
                part[r][quad] += part[r + half][quad];
            __syncthreads();
        }
        s = part[0][quad];
    }
    if (r == 0 && live)
        scale_round_store(s, alpha, beta, C + (size_t)m * ldc + n, f16, N - n < 4 ? N - n : 4);
}

}  // namespace g355

// Workspace of gemm_run_noalloc: device memory that belongs to the code object, one copy per GPU, from
// module load to process end.  In host code this name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[GEMM_NOALLOC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 16;
struct Workspace {
    void *ptr;
    size_t bytes;
};
// Registered by gemm_set_workspace, read by gemm_run: plain process-wide state, one entry per device.
// Callers that register and run from several threads order those calls themselves.
Workspace g_ws[kMaxDevices];

// Device address of `scratch` on each GPU (every GPU holds its own copy at its own address),
// looked up on the first gemm_run_noalloc call with that device current.
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];

int scratch_of_current_device(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return GEMM_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return GEMM_OK;
}

const VariantFns &launcher_of(int dtype, int id, int bl, int ragged)
{
#define G355_COUNT(...) +1
    constexpr int n_b0 = 0 G355_VARIANTS_BF16_0(G355_COUNT);
    constexpr int n_b1 = 0 G355_VARIANTS_BF16_1(G355_COUNT);
    constexpr int n_b2 = 0 G355_VARIANTS_BF16_2(G355_COUNT);
    constexpr int n_b3 = 0 G355_VARIANTS_BF16_3(G355_COUNT);
    constexpr int n_b4 = 0 G355_VARIANTS_BF16_4(G355_COUNT);
    constexpr int n_f0 = 0 G355_VARIANTS_FP8_0(G355_COUNT);
#undef G355_COUNT
    if (dtype == GEMM_FP16) {
        if (id < n_b0)
            return kLaunchFp16_0(id, bl, ragged);
        if (id < n_b0 + n_b1)
            return kLaunchFp16_1(id - n_b0, bl, ragged);
        if (id < n_b0 + n_b1 + n_b2)
            return kLaunchFp16_2(id - n_b0 - n_b1, bl, ragged);
        if (id < n_b0 + n_b1 + n_b2 + n_b3)
            return kLaunchFp16_3(id - n_b0 - n_b1 - n_b2, bl, ragged);
        if (id < n_b0 + n_b1 + n_b2 + n_b3 + n_b4)
            return kLaunchFp16_4(id - n_b0 - n_b1 - n_b2 - n_b3, bl, ragged);
        return kLaunchFp16_5(id - n_b0 - n_b1 - n_b2 - n_b3 - n_b4, bl, ragged);
    }
    if (dtype == GEMM_BF16) {
        if (id < n_b0)
            return kLaunchBf16_0(id, bl, ragged);
        if (id < n_b0 + n_b1)
            return kLaunchBf16_1(id - n_b0, bl, ragged);
        if (id < n_b0 + n_b1 + n_b2)
            return kLaunchBf16_2(id - n_b0 - n_b1, bl, ragged);
        if (id < n_b0 + n_b1 + n_b2 + n_b3)
            return kLaunchBf16_3(id - n_b0 - n_b1 - n_b2, bl, ragged);
        if (id < n_b0 + n_b1 + n_b2 + n_b3 + n_b4)
            return kLaunchBf16_4(id - n_b0 - n_b1 - n_b2 - n_b3, bl, ragged);
        return kLaunchBf16_5(id - n_b0 - n_b1 - n_b2 - n_b3 - n_b4, bl, ragged);
    }
    if (id < n_f0)
        return kLaunchFp8_0(id, bl, ragged);
    return kLaunchFp8_1(id - n_f0, bl, ragged);
}

inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }
}  // namespace

extern "C" int gemm_set_workspace(void *dev_ptr, size_t bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices)
        return GEMM_ERR_HIP;
    if (dev_ptr && ((uintptr_t)dev_ptr & 15))
        return GEMM_ERR_ALIGN;
    g_ws[dev].ptr = dev_ptr;
    g_ws[dev].bytes = dev_ptr ? bytes : 0;
    return GEMM_OK;
}

// The body of gemm_run and gemm_run_noalloc.  own_ws: nullptr = the workspace registered for the
// current device, else the buffer of own_ws_bytes bytes to use instead.
static int run_impl(const gemm_cfg *cfg, const void *A, const void *B, void *C, void *hip_stream, void *own_ws,
                    size_t own_ws_bytes)
{
    if (!cfg || !A || !B || !C)
        return GEMM_ERR_NULL;
    if (cfg->abi_version != GEMM_ABI_VERSION)
        return GEMM_ERR_ABI;
    int rc = check_problem(cfg->M, cfg->N, cfg->K, cfg->dtype);
    if (rc)
        return rc;
    const int dtype = cfg->dtype;
    const int es = elem_bytes(dtype);
    if (cfg->kernel_id < 0 || cfg->kernel_id >= variant_count(dtype))
        return GEMM_ERR_CFG_ILLEGAL;
    const Variant &v = variant_at(dtype, cfg->kernel_id);
    const gemm_hw &hw = hw_current();
    // the descriptive fields must agree with the variant the id names
    if (cfg->block_m != v.block_m || cfg->block_n != v.block_n || cfg->block_k != v.block_k ||
        cfg->waves_m != v.waves_m || cfg->waves_n != v.waves_n || cfg->mfma != v.mfma || cfg->stages != v.stages)
        return GEMM_ERR_CFG_ILLEGAL;
    if (cfg->split_k < 1 || cfg->group_m < 1 || !variant_legal(hw, v, dtype, cfg->M, cfg->N, cfg->K, cfg->split_k, 0))
        return GEMM_ERR_CFG_ILLEGAL;
    if (cfg->b_layout > 1 || cfg->stream_k > 1)
        return GEMM_ERR_CFG_ILLEGAL;
    if (cfg->groups != 0)
        return GEMM_ERR_CFG_ILLEGAL;   // a grouped cfg runs through gemm_run_grouped
    if (cfg->batch < 1 || cfg->batch > 65535)
        return GEMM_ERR_SHAPE;
    if (cfg->batch > 1 && cfg->stream_k)
        return GEMM_ERR_CFG_ILLEGAL;
    // stream-K: the plan is rebuilt from the cfg's own worker count and must exist
    SkPlan sk;
    std::memset(&sk, 0, sizeof(sk));
    if (cfg->stream_k && !cfg_stream_k_plan(cfg, &sk))
        return GEMM_ERR_CFG_ILLEGAL;
    if (cfg->lda < cfg->K || cfg->ldb < (cfg->b_layout ? cfg->K : cfg->N) || cfg->ldc < cfg->N)
        return GEMM_ERR_SHAPE;
    const int per16 = 16 / es;
    if (((uintptr_t)A & 15) || ((uintptr_t)B & 15) || ((uintptr_t)C & 15) || cfg->lda % per16 || cfg->ldb % per16 ||
        cfg->ldc % 8)
        return GEMM_ERR_ALIGN;
    if (cfg->batch > 1) {
        // problems must not overlap and must keep the 16-byte alignment of the first one
        const int64_t a_min = (cfg->M - 1) * cfg->lda + cfg->K;
        const int64_t b_min = cfg->b_layout ? (cfg->N - 1) * cfg->ldb + cfg->K : (cfg->K - 1) * cfg->ldb + cfg->N;
        const int64_t c_min = (cfg->M - 1) * cfg->ldc + cfg->N;
        if (cfg->stride_a < a_min || cfg->stride_b < b_min || cfg->stride_c < c_min)
            return GEMM_ERR_SHAPE;
        if (cfg->stride_a % per16 || cfg->stride_b % per16 || cfg->stride_c % 8)
            return GEMM_ERR_ALIGN;
        if (cfg->stride_a >= ((int64_t)1 << 40) || cfg->stride_b >= ((int64_t)1 << 40) || cfg->stride_c >= ((int64_t)1 << 40))
            return GEMM_ERR_SHAPE;
    }
    const int64_t kps = k_per_split(v, cfg->K, cfg->split_k);
    const int64_t tiles_m = cdiv64(cfg->M, v.block_m), tiles_n = cdiv64(cfg->N, v.block_n);
    // the kernel addresses a tile's operands with 32-bit byte offsets below 2 GiB
    const int64_t lim = (int64_t)1 << 31;
    const int64_t b_window = cfg->b_layout ? (int64_t)v.block_n * cfg->ldb * es
                                           : (kps + (int64_t)v.stages * v.block_k) * cfg->ldb * es;
    if ((int64_t)v.block_m * cfg->lda * es >= lim || b_window >= lim ||
        tiles_m * tiles_n * cfg->split_k + cfg->sk_workers >= lim || cfg->M * cfg->N >= ((int64_t)1 << 40))
        return GEMM_ERR_SHAPE;

    float *ws = nullptr;
    if ((cfg->split_k > 1 || cfg->stream_k) && own_ws) {
        if (own_ws_bytes < gemm_workspace_bytes(cfg))
            return GEMM_ERR_WORKSPACE;
        ws = (float *)own_ws;
    } else if (cfg->split_k > 1 || cfg->stream_k) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
            (void)hipGetLastError();
            return GEMM_ERR_HIP;
        }
        if (!g_ws[dev].ptr || g_ws[dev].bytes < gemm_workspace_bytes(cfg))
            return GEMM_ERR_WORKSPACE;
        ws = (float *)g_ws[dev].ptr;
    }

    KernelArgs a;
    a.A = A;
    a.B = B;
    a.C = C;
    a.ws = ws;
    a.M = (int)cfg->M;
    a.N = (int)cfg->N;
    a.K = (int)cfg->K;
    a.lda = (int)cfg->lda;
    a.ldb = (int)cfg->ldb;
    a.ldc = (int)cfg->ldc;
    a.alpha = cfg->alpha;
    a.beta = cfg->beta;
    a.tiles_m = (int)tiles_m;
    a.tiles_n = (int)tiles_n;
    a.split_k = cfg->split_k;
    a.k_per_split = (int)kps;
    a.group_m = (int)std::min<int64_t>(cfg->group_m, tiles_m);   // a band taller than the grid is the whole grid
    a.xcd_remap = cfg->xcd_remap ? 1 : 0;
    a.n_xcd = hw.n_xcd;
    a.sk = sk;   // workers == 0 unless stream-K
    a.batch = cfg->batch;
    a.stride_a = cfg->batch > 1 ? cfg->stride_a : 0;
    a.stride_b = cfg->batch > 1 ? cfg->stride_b : 0;
    a.stride_c = cfg->batch > 1 ? cfg->stride_c : 0;
    a.groups = nullptr;
    a.n_groups = 0;

    hipStream_t stream = (hipStream_t)hip_stream;
    const int f16 = (dtype == GEMM_FP16) ? 1 : 0;
    // an N or K that is not a whole number of 16-byte chunks runs the instantiation that trims in registers
    const int ragged = (cfg->N % per16 || cfg->K % per16) ? 1 : 0;
    // A grid of one tile row over weights larger than the memory-side cache runs the weight-streaming instantiation
    // (B's loads non-temporal, K walked in a rotated order where the weights' pitch asks for it).  Weights that fit
    // that cache are left to it: a caller that multiplies by the same weights again soon finds them there (fp8
    // M = 64, N = 28672, K = 8192, 235 MB, in a loop: 40 us cached, 48 us streamed).
    const int streaming = (!ragged && tiles_m == 1 && (double)cfg->N * (double)cfg->K * es > hw.mall_bytes) ? 2 : 0;
    if (launcher_of(dtype, cfg->kernel_id, cfg->b_layout, ragged ? 1 : streaming).launch(a, stream) != hipSuccess) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    if (cfg->stream_k) {
        // thread rows per output group: enough to keep one output's chain of contributors short
        const int contributors = sk.workers / sk.sk_tiles + 2;
        const int rows = contributors > 32 ? 8 : contributors > 8 ? 4 : 1;
        const int quads = 256 / rows;
        const int bpt = (v.block_m * v.block_n / 4 + quads - 1) / quads;
        const dim3 grid((unsigned)(sk.sk_tiles * bpt)), block(256);
        (void)hipGetLastError();
#define G355_SUM(R)                                                                                                   \
    hipLaunchKernelGGL(streamk_sum_kernel<R>, grid, block, 0, stream, ws, (uint16_t *)C, a.M, a.N, a.ldc, a.alpha,     \
                       a.beta, f16, a.tiles_m, a.tiles_n, a.group_m, sk, v.block_m, v.block_n, bpt)
        if (rows == 8)
            G355_SUM(8);
        else if (rows == 4)
            G355_SUM(4);
        else
            G355_SUM(1);
#undef G355_SUM
        if (hipGetLastError() != hipSuccess)
            return GEMM_ERR_HIP;
    } else if (cfg->split_k > 1) {
        const size_t quads = (size_t)cfg->M * (size_t)((cfg->N + 3) / 4);
        size_t blocks = (quads + 255) / 256;
        if (blocks > 256 * 8)
            blocks = 256 * 8;
        (void)hipGetLastError();
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks, (unsigned)a.batch), dim3(256), 0, stream, ws, (uint16_t *)C, a.M,
                           a.N, a.ldc, a.split_k, a.alpha, a.beta, f16, a.stride_c);
        if (hipGetLastError() != hipSuccess)
            return GEMM_ERR_HIP;
    }
    return GEMM_OK;
}

extern "C" int gemm_run(const gemm_cfg *cfg, const void *A, const void *B, void *C, void *hip_stream)
{
    return run_impl(cfg, A, B, C, hip_stream, nullptr, 0);
}

extern "C" int gemm_run_noalloc(const gemm_cfg *cfg, const void *A, const void *B, void *C, void *hip_stream)
{
    if (!cfg)
        return GEMM_ERR_NULL;
    // sizes beyond the built-in buffer are refused before anything else is looked at
    if (gemm_workspace_bytes(cfg) > (size_t)GEMM_NOALLOC_WORKSPACE_BYTES)
        return GEMM_ERR_WORKSPACE;
    void *ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc)
        return rc;
    return run_impl(cfg, A, B, C, hip_stream, ws, (size_t)GEMM_NOALLOC_WORKSPACE_BYTES);
}

extern "C" int gemm_variant_occupancy(int dtype, int variant, int b_layout, int *blocks_per_cu)
{
    if (!blocks_per_cu)
        return GEMM_ERR_NULL;
    if (dtype != GEMM_BF16 && dtype != GEMM_FP8_E4M3 && dtype != GEMM_FP16)
        return GEMM_ERR_DTYPE;
    if (variant < 0 || variant >= variant_count(dtype))
        return GEMM_ERR_INDEX;
    if (b_layout != GEMM_B_ROW_MAJOR && b_layout != GEMM_B_K_CONTIGUOUS)
        return GEMM_ERR_CFG_ILLEGAL;
    (void)hipGetLastError();
    if (launcher_of(dtype, variant, b_layout, 0).occupancy(blocks_per_cu) != hipSuccess) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    return GEMM_OK;
}

static_assert(sizeof(gemm_group_rec) == sizeof(GroupRec) && offsetof(gemm_group_rec, M) == offsetof(GroupRec, M) &&
                  offsetof(gemm_group_rec, tile_start) == offsetof(GroupRec, tile_start) &&
                  offsetof(gemm_group_rec, group_m) == offsetof(GroupRec, group_m),
              "the public record is the kernel's record");

extern "C" int gemm_run_grouped(const gemm_cfg *cfg, int n_groups, const gemm_group_rec *host_table, const void *dev_table,
                                void *hip_stream)
{
    if (!cfg || !host_table || !dev_table)
        return GEMM_ERR_NULL;
    int rc = check_grouped_cfg(cfg, n_groups);
    if (rc)
        return rc;
    if ((uintptr_t)dev_table & 15)
        return GEMM_ERR_ALIGN;
    const int X = grouped_xcds(cfg);
    int64_t slots = 0;
    int ragged = 0;   // one group with a ragged N or K sends the whole launch through the trimming instantiation
    const int per16 = 16 / elem_bytes(cfg->dtype);
    for (int i = 0; i < n_groups; ++i) {
        rc = check_group_rec(cfg, &host_table[i], slots);
        if (rc)
            return rc;
        slots += group_slots((int64_t)host_table[i].tiles_m * host_table[i].tiles_n, X);
        if (slots * X >= ((int64_t)1 << 31))
            return GEMM_ERR_SHAPE;
        if (host_table[i].M > 0 && (host_table[i].N % per16 || host_table[i].K % per16))
            ragged = 1;
    }
    if (slots == 0)
        return GEMM_OK;   // every group is empty
    const int64_t total = slots * X;
    const gemm_hw &hw = hw_current();
    KernelArgs a;
    std::memset(&a, 0, sizeof(a));
    a.alpha = cfg->alpha;
    a.beta = cfg->beta;
    a.tiles_m = (int)total;   // the grid: X workgroups per slot
    a.tiles_n = 1;
    a.split_k = 1;
    a.group_m = 1;
    a.xcd_remap = cfg->xcd_remap ? 1 : 0;
    a.n_xcd = hw.n_xcd;
    a.batch = 1;
    a.groups = (const GroupRec *)dev_table;
    a.n_groups = n_groups;
    if (launcher_of(cfg->dtype, cfg->kernel_id, cfg->b_layout, ragged).launch(a, (hipStream_t)hip_stream) != hipSuccess) {
        (void)hipGetLastError();
        return GEMM_ERR_HIP;
    }
    return GEMM_OK;
}
