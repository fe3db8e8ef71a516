// Tiled output-stationary GEMM for gfx950 (Algorithm 2 of the paper: output tiles across
// CUs in space, the reduction dimension in time; inside a tile, waves across m and n and
// MFMA k-steps in time).  One template covers the whole variant table.
//
//   A  M x K row-major, B  K x N row-major, C  M x N row-major bf16 (or fp32 partial slabs
//   when the reduction is split across workgroups).
//
// Data path per K slab: 128-bit buffer loads (A along K, B along N, out-of-range chunks
// read as zero) -> registers -> swizzled LDS (two stages) -> MFMA fragments.  A is read
// from LDS with ds_read_b128 (K-contiguous); B is N-contiguous in LDS and is read with the
// gfx950 transpose loads (ds_read_b64_tr_b16 / _tr_b8) so that each lane receives
// K-contiguous values.  The MFMA's row operand is fed from B and its column operand from
// A, so that a lane ends up with 4 consecutive n of one output row (8- or 16-byte stores).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace g355 {

struct KernelArgs {
    const void *A;
    const void *B;
    void *C;       // bf16 output (split_k == 1)
    float *ws;     // fp32 slabs [split_k][M][N] (split_k > 1)
    int M, N, K;
    int lda, ldb, ldc;  // elements
    float alpha;
    int tiles_m, tiles_n;
    int split_k;
    int k_per_split;    // elements, a multiple of BLOCK_K
    int group_m;
    int xcd_remap;
    int n_xcd;
};

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef int int2_t __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define G355_LDS __attribute__((address_space(3)))

template <int ES_, int BM_, int BN_, int BK_, int WM_, int WN_, int MI_>
struct Tile {
    static constexpr int ES = ES_, BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MI = MI_;
    static constexpr int NT = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;      // wave tile
    static constexpr int TM = WTM / MI, TN = WTN / MI;      // MFMA tiles per wave
    static constexpr int KI = (ES == 2) ? (MI == 32 ? 16 : 32) : (MI == 32 ? 64 : 128);  // MI_K
    static constexpr int KG = 64 / MI;                      // lane groups along k
    static constexpr int KL = KI / KG;                      // k elements held by one lane
    static constexpr int KSTEPS = BK / KI;
    static constexpr int RA = BK * ES;                      // bytes per A row in LDS
    static constexpr int RB = BN * ES;                      // bytes per B row in LDS
    static constexpr int A_BYTES = BM * RA, B_BYTES = BK * RB;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int ACH = A_BYTES / 16, BCH = B_BYTES / 16;  // 16-byte chunks per slab
    static constexpr int CA = RA / 16, CB = RB / 16;              // chunks per row
    static constexpr int A_LOADS = (ACH + NT - 1) / NT, B_LOADS = (BCH + NT - 1) / NT;
    static constexpr int ACC = (MI == 32) ? 16 : 4;               // fp32 accumulators per MFMA tile
    static_assert(WTM % MI == 0 && WTN % MI == 0, "wave tile must be a multiple of the MFMA tile");
    static_assert(BK % KI == 0, "BLOCK_K must be a multiple of MI_K");
    static_assert(RA % 16 == 0 && RB % 16 == 0, "rows must be whole 16-byte chunks");
    static_assert(2 * STAGE <= 160 * 1024, "two stages must fit the 160 KB LDS");

    // A rows are K-contiguous; lanes of an MFMA operand read the same chunk column of
    // consecutive rows, so the chunk index is XORed with a row key that makes 8 consecutive
    // rows land on 8 different 16-byte bank groups.
    static constexpr int A_ROWS_PER_128 = (RA >= 128) ? 1 : 128 / RA;
    static constexpr int A_KEY_MASK = ((CA < 8) ? CA : 8) - 1;
    __device__ static inline int a_off(int row, int chunk) {
        int key = (row / A_ROWS_PER_128) & A_KEY_MASK;
        return row * RA + ((chunk ^ key) << 4);
    }
    // B rows are N-contiguous; a transpose read touches SEG bytes of each of several
    // consecutive k rows, so the SEG-sized block index inside a row is XORed with a key of k
    // that spreads consecutive rows over 256 bytes of banks.
    static constexpr int SEG_BITS = (ES == 2) ? 6 : 5;
    static constexpr int SEG = 1 << SEG_BITS;
    static constexpr int B_SPREAD = 256 / SEG;
    static constexpr int B_ROW_DIV = (RB >= 256) ? 1 : 256 / RB;
    static constexpr int B_KEY_MASK = (((RB / SEG) < B_SPREAD) ? ((RB / SEG) > 0 ? (RB / SEG) : 1) : B_SPREAD) - 1;
    __device__ static inline int b_off(int krow, int nbyte) {
        int key = (krow / B_ROW_DIV) & B_KEY_MASK;
        return krow * RB + (nbyte ^ (key << SEG_BITS));
    }
};

// Workgroup id -> (tile_m, tile_n, k_slice).  Hardware deals consecutive workgroup ids
// round-robin to the XCDs; the remap gives every XCD one contiguous range of logical ids,
// and inside the tile grid the ids run column-major through bands of group_m tile rows,
// so the workgroups that share an L2 at one time form a compact group_m x (CUs/group_m)
// block of output tiles (the cache tile of Algorithms 5 and 6).
__device__ inline void tile_coords(const KernelArgs &a, int pid, int &tm, int &tn, int &ks)
{
    const int tiles = a.tiles_m * a.tiles_n;
    int l = pid;
    if (a.xcd_remap) {
        const int grid = tiles * a.split_k;
        const int per = grid / a.n_xcd, rem = grid % a.n_xcd;
        const int x = pid % a.n_xcd, q = pid / a.n_xcd;
        l = x * per + (x < rem ? x : rem) + q;
    }
    ks = l / tiles;
    const int t = l - ks * tiles;
    const int band_sz = a.group_m * a.tiles_n;
    const int band = t / band_sz;
    const int first_m = band * a.group_m;
    const int rows = (a.tiles_m - first_m < a.group_m) ? (a.tiles_m - first_m) : a.group_m;
    const int r = t - band * band_sz;
    tm = first_m + r % rows;
    tn = r / rows;
}

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    // raw buffer window [base, base + bytes): loads at offsets reaching beyond it return zero
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// beyond every window (windows are validated to stay below 2 GiB); small advances keep it there
constexpr unsigned OOB_OFFSET = 0x80000000u;

template <class T>
__global__ __launch_bounds__(T::NT) void gemm_kernel(const KernelArgs args)
{
    constexpr int ES = T::ES, BM = T::BM, BN = T::BN, BK = T::BK, MI = T::MI, NT = T::NT;
    __shared__ __attribute__((aligned(128))) uint8_t smem[2 * T::STAGE];

    int tm, tn, ks;
    tile_coords(args, blockIdx.x, tm, tn, ks);
    const int m0 = tm * BM, n0 = tn * BN;
    const int k_begin = ks * args.k_per_split;
    int k_len = args.K - k_begin;
    if (k_len > args.k_per_split)
        k_len = args.k_per_split;
    const int kt_count = (k_len + BK - 1) / BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / T::WN, wn = wave % T::WN;

    // ---- global load bookkeeping ----
    // Chunk c (16 bytes) of a slab belongs to thread c % NT; NT is a multiple of the chunks
    // per row, so a thread keeps one chunk column and steps down the rows.  Rows past the
    // edge of the matrix (A: m >= M, B: k >= k_len) fall outside the buffer window and read
    // as zero; chunk columns past the edge (A: k >= k_len, B: n >= N) are sent there by
    // replacing the offset.
    static_assert(NT % T::CA == 0 && NT % T::CB == 0, "a thread must keep one chunk column");
    constexpr int A_RSTEP = NT / T::CA, B_RSTEP = NT / T::CB;
    const uint8_t *Abase = (const uint8_t *)args.A + ((size_t)m0 * args.lda + k_begin) * ES;
    const uint8_t *Bbase = (const uint8_t *)args.B + ((size_t)k_begin * args.ldb + n0) * ES;
    const int a_rows_valid = (args.M - m0 < BM) ? (args.M - m0) : BM;
    const __amdgpu_buffer_rsrc_t rsA =
        make_rsrc(Abase, (unsigned)((a_rows_valid - 1) * args.lda + k_len) * ES);
    const __amdgpu_buffer_rsrc_t rsB = make_rsrc(Bbase, (unsigned)(k_len * args.ldb) * ES);

    const int a_row0 = tid / T::CA, a_ch = tid % T::CA;
    const int b_row0 = tid / T::CB, b_ch = tid % T::CB;
    const int a_kcol = a_ch * (16 / ES);
    const bool a_active = a_row0 < BM;
    const bool b_active = (b_row0 < BK) && (n0 + b_ch * (16 / ES) < args.N);
    const unsigned a_voff0 = a_active ? (unsigned)(a_row0 * args.lda * ES + a_ch * 16) : OOB_OFFSET;
    const unsigned b_voff0 = b_active ? (unsigned)(b_row0 * args.ldb * ES + b_ch * 16) : OOB_OFFSET;
    const unsigned a_rstep = (unsigned)(A_RSTEP * args.lda * ES);
    const unsigned b_rstep = (unsigned)(B_RSTEP * args.ldb * ES);

    i32x4 a_reg[T::A_LOADS], b_reg[T::B_LOADS];
    auto load_slab = [&](int kt) {
        const int kk = kt * BK;
        const unsigned a_base = (a_kcol + kk < k_len) ? a_voff0 + (unsigned)(kk * ES) : OOB_OFFSET;
        const unsigned b_base = b_voff0 + (unsigned)kk * (unsigned)(args.ldb * ES);
#pragma unroll
        for (int i = 0; i < T::A_LOADS; ++i)
            a_reg[i] = __builtin_bit_cast(
                i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsA, a_base + i * a_rstep, 0, 0));
#pragma unroll
        for (int i = 0; i < T::B_LOADS; ++i)
            b_reg[i] = __builtin_bit_cast(
                i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsB, b_base + i * b_rstep, 0, 0));
    };
    auto store_slab = [&](int stage) {
        uint8_t *s = smem + stage * T::STAGE;
#pragma unroll
        for (int i = 0; i < T::A_LOADS; ++i)
            if (T::ACH >= NT || a_row0 < BM)
                *(i32x4 *)(s + T::a_off(a_row0 + i * A_RSTEP, a_ch)) = a_reg[i];
#pragma unroll
        for (int i = 0; i < T::B_LOADS; ++i)
            if (T::BCH >= NT || b_row0 < BK)
                *(i32x4 *)(s + T::A_BYTES + T::b_off(b_row0 + i * B_RSTEP, b_ch * 16)) = b_reg[i];
    };

    // ---- fragment addressing (per lane, constant over the K loop) ----
    // column operand (from A): lane holds row m = lane % MI, k in [kg*KL, kg*KL + KL)
    const int a_row = wm * T::WTM + (lane % MI);
    const int a_kg = lane / MI;
    // row operand (from B, transposed): 16-lane group g, lane i of it supplies the address of
    // k row (i / LPR) and n block (i % LPR); it receives n = i, k = 0 .. 64/16*ES ... of the group
    const int g16 = lane >> 4, i16 = lane & 15;
    const int b_nhalf = (MI == 32) ? (g16 & 1) : 0;
    const int b_kg = (MI == 32) ? (g16 >> 1) : g16;
    constexpr int LPR = (ES == 2) ? 4 : 2;          // lanes that share one k row in a transpose read
    constexpr int TRK = 16 / LPR;                   // k rows covered by one transpose read (4 or 8)
    const int b_krow_l = b_kg * T::KL + i16 / LPR;
    const int b_ncol = wn * T::WTN + b_nhalf * 16 + (i16 % LPR) * (8 / ES);   // element column

    typedef typename std::conditional<MI == 32, f32x16, f32x4>::type acc_t;
    acc_t acc[T::TN][T::TM];
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
        for (int i = 0; i < T::TM; ++i)
#pragma unroll
            for (int r = 0; r < T::ACC; ++r)
                acc[j][i][r] = 0.f;

    auto compute = [&](int stage) {
        const uint8_t *sA = smem + stage * T::STAGE;
        const uint8_t *sB = sA + T::A_BYTES;
#pragma unroll
        for (int kstep = 0; kstep < T::KSTEPS; ++kstep) {
            const int k0 = kstep * T::KI;
            if constexpr (ES == 2) {
                bf16x8 af[T::TM], bfr[T::TN];
#pragma unroll
                for (int i = 0; i < T::TM; ++i) {
                    const int chunk = (k0 + a_kg * T::KL) / 8;
                    af[i] = *(const bf16x8 *)(sA + T::a_off(a_row + i * MI, chunk));
                }
#pragma unroll
                for (int j = 0; j < T::TN; ++j) {
                    short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (G355_LDS short4_t *)(sB + T::b_off(k0 + b_krow_l, (b_ncol + j * MI) * 2)));
                    short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (G355_LDS short4_t *)(sB + T::b_off(k0 + b_krow_l + TRK, (b_ncol + j * MI) * 2)));
                    typedef short short8_t __attribute__((ext_vector_type(8)));
                    short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    bfr[j] = __builtin_bit_cast(bf16x8, v);
                }
#pragma unroll
                for (int j = 0; j < T::TN; ++j)
#pragma unroll
                    for (int i = 0; i < T::TM; ++i) {
                        if constexpr (MI == 32)
                            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[j][i], 0, 0, 0);
                        else
                            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j], af[i], acc[j][i], 0, 0, 0);
                    }
            } else {
                i32x8 af[T::TM], bfr[T::TN];
#pragma unroll
                for (int i = 0; i < T::TM; ++i) {
                    const int chunk = (k0 + a_kg * T::KL) / 16;
                    i32x4 lo = *(const i32x4 *)(sA + T::a_off(a_row + i * MI, chunk));
                    i32x4 hi = *(const i32x4 *)(sA + T::a_off(a_row + i * MI, chunk + 1));
                    af[i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int j = 0; j < T::TN; ++j) {
                    int2_t q[4];
#pragma unroll
                    for (int h = 0; h < 4; ++h)
                        q[h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                            (G355_LDS int2_t *)(sB + T::b_off(k0 + b_krow_l + h * TRK, b_ncol + j * MI)));
                    i32x4 lo = __builtin_shufflevector(q[0], q[1], 0, 1, 2, 3);
                    i32x4 hi = __builtin_shufflevector(q[2], q[3], 0, 1, 2, 3);
                    bfr[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int j = 0; j < T::TN; ++j)
#pragma unroll
                    for (int i = 0; i < T::TM; ++i) {
                        if constexpr (MI == 32)
                            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bfr[j], af[i], acc[j][i], 0, 0, 0, 0, 0, 0);
                        else
                            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bfr[j], af[i], acc[j][i], 0, 0, 0, 0, 0, 0);
                    }
            }
        }
    };

    // ---- pipeline: prologue, main K loop, epilogue (Algorithm 8's three phases) ----
    if (kt_count > 0) {
        load_slab(0);
        store_slab(0);
    }
    __syncthreads();
    for (int kt = 0; kt < kt_count; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < kt_count;
        if (more)
            load_slab(kt + 1);
        compute(cur);
        if (more)
            store_slab(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds, per MFMA tile, output row m = lane % MI and
    //      n = 8*(r/4) + 4*(lane/32) + r%4 (32x32) or n = 4*(lane/16) + r (16x16) ----
    const int out_m = m0 + wm * T::WTM + (lane % MI);
    const int out_nl = n0 + wn * T::WTN + 4 * (lane / MI);
    const float alpha = args.alpha;
#pragma unroll
    for (int i = 0; i < T::TM; ++i) {
        const int m = out_m + i * MI;
        if (m >= args.M)
            continue;
#pragma unroll
        for (int j = 0; j < T::TN; ++j) {
#pragma unroll
            for (int q = 0; q < T::ACC / 4; ++q) {
                const int n = out_nl + j * MI + q * 8;
                if (n >= args.N)
                    continue;
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = acc[j][i][q * 4 + r];
                if (args.split_k > 1) {
                    float *dst = args.ws + ((size_t)ks * args.M + m) * args.N + n;
                    *(f32x4 *)dst = v;
                } else {
                    bf16x4 o;
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        o[r] = (__bf16)(v[r] * alpha);
                    __bf16 *dst = (__bf16 *)args.C + (size_t)m * args.ldc + n;
                    *(bf16x4 *)dst = o;
                }
            }
        }
    }
}

}  // namespace g355
