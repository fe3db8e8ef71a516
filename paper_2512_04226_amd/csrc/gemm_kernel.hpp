// Tiled output-stationary GEMM for gfx950 (Algorithm 2 of the paper: output tiles across
// CUs in space, the reduction dimension in time; inside a tile, waves across m and n and
// MFMA k-steps in time).  One template covers the whole variant table.
//
//   A  M x K row-major, B  K x N row-major (or N x K row-major, K-contiguous), C  M x N
//   row-major bf16 (fp16 for fp16 inputs), or fp32 partials when the reduction of a tile is
//   shared between workgroups (split-K slabs, Stream-K partial tiles).  blockIdx.y selects
//   the problem of a strided batch.
//
// Data path per K slab: 128-bit buffer loads straight into LDS (A along K, B along N or K,
// out-of-range chunks arrive as zero; no register staging) -> swizzled LDS ring of NS
// stages -> MFMA fragments.  A is read from LDS with ds_read_b128 (K-contiguous); row-major
// B is N-contiguous in LDS and is read with the gfx950 transpose loads (ds_read_b64_tr_b16 /
// _tr_b8) so that each lane receives K-contiguous values; K-contiguous B is read like A.
// The MFMA's row operand is fed from B and its column operand from A, so that a lane ends
// up with 4 consecutive n of one output row (8- or 16-byte stores).
//
// A workgroup computes one (tile, K slice), or -- as a Stream-K worker -- up to two
// (tile, slab range) segments, with the same prologue / K loop / epilogue body.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "grouped.hpp"
#include "stream_k.hpp"

namespace g355 {

struct KernelArgs {
    const void *A;
    const void *B;
    void *C;       // bf16 (fp16 for fp16 inputs) output
    float *ws;     // fp32 slabs [split_k][M][N] (split_k > 1), or stream-K partial tiles
    int M, N, K;
    int lda, ldb, ldc;  // elements
    float alpha, beta;  // C = alpha*A*B + beta*C; beta == 0: C is not read
    int tiles_m, tiles_n;
    int split_k;
    int k_per_split;    // elements, a multiple of BLOCK_K
    int group_m;
    int xcd_remap;
    int n_xcd;
    // Stream-K (sk.workers > 0, split_k == 1): workgroups [0, sk.workers) are stream-K workers,
    // the rest compute the sk.dp_tiles data-parallel tiles; ws then holds the workers' partial
    // tiles, [2 * workers][BLOCK_M][BLOCK_N] fp32.
    SkPlan sk;
    // Strided batch: blockIdx.y selects the problem; strides in elements (the workspace of
    // problem b starts at b * split_k * M * N floats).
    long long stride_a, stride_b, stride_c;
    int batch;
    // Grouped launch (n_groups > 0; split_k == 1, no stream-K, batch == 1): the problem fields
    // above are unused and each workgroup reads its group's record from this device table.
    const GroupRec *groups;
    int n_groups;
};

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef int int2_t __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define G355_LDS __attribute__((address_space(3)))
// K-loop form 5's scheduling fence after MFMA m of a k-step
#ifndef G355_LF5_EVERY
#define G355_LF5_EVERY 1
#endif
#ifndef G355_LF5_MASK
#define G355_LF5_MASK 0
#endif
#define G355_LF5_FENCE(m)                                      \
    do {                                                       \
        if ((m) % G355_LF5_EVERY == G355_LF5_EVERY - 1)        \
            __builtin_amdgcn_sched_barrier(G355_LF5_MASK);     \
    } while (0)
// Cache-policy operand of the slab loads: 0 = default, 2 = the instruction's `nt` (non-temporal) modifier.
#define G355_LOAD_DEFAULT 0
#define G355_LOAD_STREAM 2

// BL_: storage of B.  0: K x N row-major (N-contiguous).  1: N x K row-major (K-contiguous, the
// layout of the paper's own runs, Section V): B is then staged and read exactly like A.
// FT_ (16-bit inputs only): 0 bf16 in / bf16 out, 1 IEEE fp16 in / fp16 out (the precision of the
// paper's runs); the data path is the same, only the MFMA instruction and the output rounding differ.
// LF_: form of the K loop, one of seven source arrangements of the same work between which the
// compiler's instruction schedule, and with it the time per slab, differs by up to 15 % either
// way; which one a variant uses is measured (8192^3, the forms interleaved) and recorded
// in the variant table.  0: one loop over all slabs, the part up to the next barrier under a
// condition that is false for the last slab.  1: the last slab peeled off, so the first fragment
// reads of the next slab cannot sink into a conditional part below the MFMAs meant to hide them.
// 2: as 1, and no memory instruction may be scheduled across the end of the refill (the refill
// of the freed stage goes out first: it has the fewest iterations to land in a two-stage ring).
// 3: as 1, with the order of every k-step's memory and matrix instructions prescribed: after the
// barrier the refill two loads per MFMA, then in each k-step the fragment reads of the next one a
// few per MFMA over the first half of its MFMAs, so that a read has half a k-step to land (the
// compiler alone issues reads next to their uses, which costs most with one wave per SIMD).
// 4: as 3, but the refill is spread evenly over ALL the MFMAs of the k-step after the barrier (one load every
// MN / NL matrix instructions) instead of going out as a burst: the vector-memory path of a CU takes 64 bytes
// per clock, a slab's loads are 16 clocks of it each, and a wave whose load finds that path's queue full
// cannot issue the MFMAs behind it either.
// 5: the order written out in the source instead of prescribed to the scheduler: every MFMA of a k-step is preceded
// by its share of the refill loads (after the barrier) and of the next k-step's fragment reads (first half of the
// MFMAs), and a scheduling fence after each MFMA keeps the compiler from moving anything across it.  Both fragment
// buffers are then live through every k-step: the four-wave tiles and several medium tiles gain 3-13 %, the 256x256
// eight-wave tiles on a 4x2 grid would spill.
// 6: only the A fragments are double-buffered; the B fragments pass through a ring of four register slots that is
// read three (k-step, column) blocks ahead of the MFMAs, and the slab's barrier follows the last fragment read of
// the stage, not its last MFMA.  Fewer live registers than form 5 (the eight-wave 256x256x64 tiles keep no spills);
// needs three or more column blocks per wave and a multiple of four blocks per slab, else the tile runs form 0.
// Building with -DG355_FORCE_LOOP_FORM=k gives every variant form k (how the forms are compared).
// Timing-only diagnostic builds (their RESULTS ARE WRONG; every access stays in bounds and every wait ends):
// -DG355_DIAG_SKIP_FILL leaves the refills out of the K loop (the ring keeps its first NS slabs),
// -DG355_DIAG_SKIP_FRAG the fragment reads (the MFMAs reuse the first slab's fragments), -DG355_DIAG_SKIP_MFMA the
// matrix instructions; timed against a normal build they show what the fill, the LDS reads and the MFMAs cost a
// slab on their own and together (calibrate.py --decompose).  -DG355_DIAG_PANEL=b lets every workgroup read the
// A rows of tile row 0 (bit 0) and the B columns of tile column 0 (bit 1; with bit 2: of tile row / column
// blockIdx % 8), so that every request hits in the L2; -DG355_DIAG_FILL_MODE=1 sends the refill into registers
// that nothing reads (no LDS writes), =2 issues the same requests 4 bytes per lane instead of 16
// (calibrate.py --compare-builds; run them on shapes that are whole tiles and whole slabs only).
// RG_: 1 = the instantiation for shapes whose N or K is not a whole number of 16-byte chunks.  A chunk that
// holds the end of a row of a K-contiguous operand then also holds bytes that are not part of the matrix
// (padding up to the leading dimension, which may be anything, NaN included), so slabs go through registers,
// where those elements are cleared, and are written to LDS with ds_write_b128 (a plain two-stage loop: the
// next slab's global loads fly during the current slab's MFMAs); results at the ragged edge of C are stored
// element by element.  Everything else -- LDS layout, fragments, MFMAs, staged epilogue -- is shared.
// ST_: 1 = the weight-streaming instantiation for grids of one tile row (see STREAMABLE_B in Tile).
template <int ES_, int BM_, int BN_, int BK_, int WM_, int WN_, int MI_, int NS_, int BL_, int FT_ = 0, int LF_ = 0, int RG_ = 0, int ST_ = 0>
struct Tile {
    static constexpr int ES = ES_, BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MI = MI_, NS = NS_, BL = BL_;
    static constexpr int FT = FT_;
    static constexpr int RG = RG_;
    static constexpr int ST = ST_;
#ifdef G355_FORCE_LOOP_FORM
    static constexpr int LF_ASKED = G355_FORCE_LOOP_FORM;
#else
    static constexpr int LF_ASKED = LF_;
#endif
    static_assert(LF_ASKED >= 0 && LF_ASKED <= 6, "unknown K-loop form");
    static_assert(FT == 0 || ES == 2, "fp16 is a 16-bit input type");
    static constexpr int NW = WM * WN;
    static constexpr int NT = WM * WN * 64;
    // ST_ = 1: the weight-streaming instantiation, which the host launches for a grid of one tile row (M <= BLOCK_M)
    // over weights larger than the memory-side cache.  Every byte of B is then read once: its slab loads carry the non-temporal
    // hint, so that the stream does not push A's panel, which every workgroup re-reads, out of the L2 (5-10 % on
    // the HBM-bound shapes), and K-contiguous weights with a power-of-two row pitch are walked in a rotated order
    // (see `rot` in gemm_kernel).  The cache policy is an immediate of the load instruction and the rotation a
    // few scalar instructions per slab; as a second copy of the loop inside one kernel either cost the other copy
    // registers or its schedule (128x128x64: a resident workgroup, or 2-12 % on every other shape), so the
    // streaming loop is a kernel of its own.
    static constexpr bool STREAMABLE_B = ST == 1, STREAMABLE_A = false;
    static constexpr int WTM = BM / WM, WTN = BN / WN;      // wave tile
    static constexpr int TM = WTM / MI, TN = WTN / MI;      // MFMA tiles per wave
    static constexpr int KI = (ES == 2) ? (MI == 32 ? 16 : 32) : (MI == 32 ? 64 : 128);  // MI_K
    static constexpr int KG = 64 / MI;                      // lane groups along k
    static constexpr int KL = KI / KG;                      // k elements held by one lane
    static constexpr int KSTEPS = BK / KI;
    // form 6 needs at least three B fragments per k-step and a whole number of four-slot ring turns per slab;
    // a tile that has neither runs form 0 when form 6 is forced on every tile
    static constexpr int LF = (LF_ASKED == 6 && !(TN >= 3 && (KSTEPS * TN) % 4 == 0 && KSTEPS >= 2)) ? 0 : LF_ASKED;
    static constexpr int RA = BK * ES;                      // bytes per A row in LDS
    static constexpr int RB = (BL == 0) ? BN * ES : BK * ES; // bytes per B row in LDS (a k row, or an n row when K-contiguous)
    static constexpr int A_BYTES = BM * RA, B_BYTES = BK * BN * ES;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int ACH = A_BYTES / 16, BCH = B_BYTES / 16;  // 16-byte chunks per slab
    static constexpr int CA = RA / 16, CB = RB / 16;              // chunks per row
    // a direct-to-LDS load instruction of one wave fills one 1 KB unit (64 lanes x 16 bytes)
    static constexpr int A_UNITS = ACH / 64, B_UNITS = BCH / 64;
    static constexpr int A_LOADS = (A_UNITS + NW - 1) / NW, B_LOADS = (B_UNITS + NW - 1) / NW;
    static_assert(ACH % 64 == 0 && BCH % 64 == 0, "slabs must be whole 1 KB units");
    // does every wave of the workgroup issue load instruction l of a slab request?
    static constexpr bool every_wave_issues(int l) {
        return (l < A_LOADS) ? (A_UNITS % NW == 0 || (l * NW + NW - 1) < A_UNITS)
                             : (B_UNITS % NW == 0 || ((l - A_LOADS) * NW + NW - 1) < B_UNITS);
    }
    static constexpr int common_loads() {   // load instructions of a slab request that every wave issues
        int full = 0;
        for (int l = 0; l < A_LOADS + B_LOADS; ++l)
            if (every_wave_issues(l))
                ++full;
        return full;
    }
    static constexpr int ACC = (MI == 32) ? 16 : 4;               // fp32 accumulators per MFMA tile
    static_assert(WTM % MI == 0 && WTN % MI == 0, "wave tile must be a multiple of the MFMA tile");
    static_assert(BK % KI == 0, "BLOCK_K must be a multiple of MI_K");
    static_assert(RA % 16 == 0 && RB % 16 == 0, "rows must be whole 16-byte chunks");
    static_assert(NS >= 2 && NS * STAGE <= 160 * 1024, "the stage ring must fit the 160 KB LDS");

    // A rows are K-contiguous; the lanes of an MFMA operand read the same chunk column of
    // consecutive rows.  The LDS has 64 four-byte banks (256 bytes per clock) and serves a
    // ds_read_b128 sixteen lanes at a time, so sixteen consecutive rows must land on sixteen
    // different 16-byte slots of the 256-byte bank window: the chunk index is XORed with a key
    // that counts 256-byte windows of rows.
    static constexpr int A_ROWS_PER_WIN = (RA >= 256) ? 1 : 256 / RA;
    static constexpr int A_KEY_MASK = ((CA < 16) ? CA : 16) - 1;
    __device__ static inline int a_key(int row) { return (row / A_ROWS_PER_WIN) & A_KEY_MASK; }
    __device__ static inline int a_off(int row, int chunk) { return row * RA + ((chunk ^ a_key(row)) << 4); }
    // B rows are N-contiguous; a transpose read touches SEG bytes of each of several
    // consecutive k rows, so the SEG-sized block index inside a row is XORed with a key of k
    // that spreads consecutive rows over 256 bytes of banks.  With the 16x16 MFMA the two
    // 16-lane groups that are served together read the same 32 bytes of k rows 8 apart, so
    // for 16-bit types the 32-byte half inside a segment is flipped by bit 3 of k as well
    // (a no-op for the 32x32 pattern, whose paired groups already differ by 32 bytes of n).
    static constexpr int SEG_BITS = (ES == 2) ? 6 : 5;
    static constexpr int SEG = 1 << SEG_BITS;
    static constexpr int B_SPREAD = 256 / SEG;
    static constexpr int B_ROW_DIV = (RB >= 256) ? 1 : 256 / RB;
    static constexpr int B_KEY_MASK = (((RB / SEG) < B_SPREAD) ? ((RB / SEG) > 0 ? (RB / SEG) : 1) : B_SPREAD) - 1;
    static constexpr int B_HALF_FLIP = (ES == 2 && RB >= 64) ? 32 : 0;
    __device__ static inline int b_key(int krow)
    {
        return (((krow / B_ROW_DIV) & B_KEY_MASK) << SEG_BITS) ^ (((krow >> 3) & 1) * B_HALF_FLIP);
    }
    __device__ static inline int b_off(int krow, int nbyte) { return krow * RB + (nbyte ^ b_key(krow)); }
};

// Workgroup id -> (tile_m, tile_n, k_slice).  Hardware deals consecutive workgroup ids
// round-robin to the XCDs; the remap gives every XCD one contiguous range of logical ids,
// and inside the tile grid the ids run column-major through bands of group_m tile rows,
// so the workgroups that share an L2 at one time form a compact group_m x (CUs/group_m)
// block of output tiles (the cache tile of Algorithms 5 and 6).
// pid in [0, grid), grid = data-parallel tiles * split_k.
__device__ inline int logical_id(const KernelArgs &a, int pid, int grid)
{
    if (!a.xcd_remap)
        return pid;
    const int per = grid / a.n_xcd, rem = grid % a.n_xcd;
    const int x = pid % a.n_xcd, q = pid / a.n_xcd;
    return x * per + (x < rem ? x : rem) + q;
}

__device__ inline void tile_coords(const KernelArgs &a, int pid, int grid, int &tm, int &tn, int &ks)
{
    const int tiles = a.tiles_m * a.tiles_n;
    const int l = logical_id(a, pid, grid);
    ks = l / tiles;
    logical_tile(a.tiles_m, a.tiles_n, a.group_m, l - ks * tiles, tm, tn);
}

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    // raw buffer window [base, base + bytes): loads at offsets reaching beyond it return zero
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// beyond every window (windows are validated to stay below 2 GiB); small advances keep it there
constexpr unsigned OOB_OFFSET = 0x80000000u;

// Scheduling pipelines of K-loop form 3: COUNT times "A LDS reads (or A global loads), then one
// MFMA".  The calls follow the code they order: a group takes the nearest matching instructions
// before it, so the counts of a pipeline add up to exactly the instructions of its k-step.
// Group masks: 0x008 matrix instructions, 0x020 vector-memory loads, 0x100 LDS reads.
template <int COUNT, int A>
__device__ __forceinline__ void sched_reads_then_mfma()
{
    if constexpr (COUNT > 0) {
        __builtin_amdgcn_sched_group_barrier(0x100, A, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        sched_reads_then_mfma<COUNT - 1, A>();
    }
}
template <int COUNT, int A>
__device__ __forceinline__ void sched_fills_then_mfma()
{
    if constexpr (COUNT > 0) {
        __builtin_amdgcn_sched_group_barrier(0x020, A, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        sched_fills_then_mfma<COUNT - 1, A>();
    }
}

// K-loop form 4, the k-step after the barrier: MFMA number I of MN is preceded by its even share of the NL
// refill loads and, in the first half, of the NFR fragment reads.
template <int I, int MN, int NL, int NFR>
__device__ __forceinline__ void sched_spread_fills()
{
    if constexpr (I < MN) {
        constexpr int H = MN > 1 ? MN / 2 : 1;
        constexpr int loads = (I + 1) * NL / MN - I * NL / MN;
        constexpr int reads = I < H ? (I + 1) * NFR / H - I * NFR / H : 0;
        if constexpr (loads > 0)
            __builtin_amdgcn_sched_group_barrier(0x020, loads, 0);
        if constexpr (reads > 0)
            __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        sched_spread_fills<I + 1, MN, NL, NFR>();
    }
}

template <class T>
__global__ __launch_bounds__(T::NT) void gemm_kernel(const KernelArgs args)
{
    constexpr int ES = T::ES, BM = T::BM, BN = T::BN, BK = T::BK, MI = T::MI;
    __shared__ __attribute__((aligned(1024))) uint8_t smem[T::NS * T::STAGE];

    // Work of this workgroup: one (tile, K slice) for a data-parallel or split-K launch, up to
    // two (tile, slab range) segments for a stream-K worker.
    const bool sk_worker = (int)blockIdx.x < args.sk.workers;
    SkSegment segs[2];
    int nseg = 1;
    if (sk_worker)
        nseg = sk_segments(args.sk, (int)blockIdx.x, segs);

    // The problem this workgroup works on: the launch's own, or its group's in a grouped launch.
    const void *pA = args.A, *pB = args.B;
    void *pC = args.C;
    int pM = args.M, pN = args.N, pK = args.K, plda = args.lda, pldb = args.ldb, pldc = args.ldc;
    int g_tm = 0, g_tn = 0;
    const bool grouped = args.n_groups > 0;
    // one tile row: B is read once; one tile column: A is read once (see Tile::STREAMABLE_*)
    bool stream_a = args.tiles_n == 1, stream_b = T::ST == 1;
    if (grouped) {
        const int X = args.xcd_remap ? args.n_xcd : 1;
        const int x = (int)blockIdx.x % X, q = (int)blockIdx.x / X;
        const GroupRec *r = args.groups + group_of(args.groups, args.n_groups, q);
        const int tiles_m = uniform_i32(r->tiles_m), tiles_n = uniform_i32(r->tiles_n);
        stream_a = tiles_n == 1;
        const int t = group_tile(tiles_m * tiles_n, X, x, q - uniform_i32(r->tile_start));
        if (t < 0)
            return;   // idle slot of this XCD (the whole workgroup leaves: nothing was started)
        pA = uniform_ptr(r->A);
        pB = uniform_ptr(r->B);
        pC = uniform_ptr(r->C);
        pM = uniform_i32(r->M);
        pN = uniform_i32(r->N);
        pK = uniform_i32(r->K);
        plda = uniform_i32(r->lda);
        pldb = uniform_i32(r->ldb);
        pldc = uniform_i32(r->ldc);
        logical_tile(tiles_m, tiles_n, uniform_i32(r->group_m), t, g_tm, g_tn);
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept scalar
    const int wm = wave / T::WN, wn = wave % T::WN;

    for (int seg = 0; seg < nseg; ++seg) {
    // out_mode 0: bf16 C;  1: fp32 split-K slab ks;  2: fp32 partial tile of a stream-K segment
    int tm, tn, ks = 0, k_begin, k_len, out_mode;
    if (sk_worker) {
        const SkSegment sg = (seg == 0) ? segs[0] : segs[1];
        logical_tile(args.tiles_m, args.tiles_n, args.group_m, args.sk.dp_tiles + sg.tile, tm, tn);
        k_begin = sg.slab0 * BK;
        k_len = sg.count * BK;
        if (k_len > pK - k_begin)
            k_len = pK - k_begin;
        out_mode = sg.complete ? 0 : 2;
        if (seg) {
            // the previous segment's stores have left and every wave is done with its LDS stages
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    } else if (grouped) {
        tm = g_tm;
        tn = g_tn;
        k_begin = 0;
        k_len = pK;
        out_mode = 0;
    } else {
        const int grid = (args.sk.workers > 0) ? args.sk.dp_tiles : args.tiles_m * args.tiles_n * args.split_k;
        tile_coords(args, (int)blockIdx.x - args.sk.workers, grid, tm, tn, ks);
        k_begin = ks * args.k_per_split;
        k_len = pK - k_begin;
        if (k_len > args.k_per_split)
            k_len = args.k_per_split;
        out_mode = (args.split_k > 1) ? 1 : 0;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int kt_count = (k_len + BK - 1) / BK;

    // ---- global -> LDS bookkeeping ----
    // Load instruction i of wave w fills LDS unit u = i*NW + w of the stage: lane l writes the
    // 16-byte slot c = u*64 + l (row c / chunks-per-row, physical chunk c % chunks-per-row).
    // The swizzle is applied on the global side: the lane fetches the logical chunk that
    // belongs in its slot.  Rows past the edge of the matrix (A: m >= M, B: k >= k_len) fall
    // outside the buffer window and arrive as zero; chunk columns past the edge (A: k >= k_len,
    // B: n >= N) are sent outside the window by replacing the offset.
    const size_t bz = blockIdx.y;     // problem of the batch
#ifdef G355_DIAG_PANEL
    // timing-only builds: every workgroup (bit 0: of an XCD, with bit 2) reads the A rows of tile row 0,
    // (bit 1) the B columns of tile column 0 -- the results are wrong, the request stream keeps its shape
    const int m0_ld = (G355_DIAG_PANEL & 1) ? ((G355_DIAG_PANEL & 4) ? (int)(blockIdx.x % 8) * BM : 0) : m0;
    const int n0_ld = (G355_DIAG_PANEL & 2) ? ((G355_DIAG_PANEL & 4) ? (int)(blockIdx.x % 8) * BN : 0) : n0;
#else
    const int m0_ld = m0, n0_ld = n0;
#endif
    const uint8_t *Abase = (const uint8_t *)pA + (bz * args.stride_a + (size_t)m0_ld * plda + k_begin) * ES;
    const uint8_t *Bbase = (T::BL == 0)
                               ? (const uint8_t *)pB + (bz * args.stride_b + (size_t)k_begin * pldb + n0_ld) * ES
                               : (const uint8_t *)pB + (bz * args.stride_b + (size_t)n0_ld * pldb + k_begin) * ES;
    const int a_rows_valid = (pM - m0 < BM) ? (pM - m0) : BM;
    const int b_rows_valid = (pN - n0 < BN) ? (pN - n0) : BN;      // K-contiguous B only
    // (ragged instantiation: the window ends with the chunk that holds the last valid element, so that this
    // chunk is fetched whole and trimmed in registers; rows are a whole number of chunks apart, so it lies
    // inside the last row's leading-dimension span)
    constexpr int EPC = 16 / ES;                                   // elements per 16-byte chunk
    const int k_len_w = T::RG ? (k_len + EPC - 1) / EPC * EPC : k_len;
    const __amdgpu_buffer_rsrc_t rsA =
        make_rsrc(Abase, (unsigned)((a_rows_valid - 1) * plda + k_len_w) * ES);
    const __amdgpu_buffer_rsrc_t rsB =
        make_rsrc(Bbase, (T::BL == 0) ? (unsigned)(k_len * pldb) * ES
                                      : (unsigned)((b_rows_valid - 1) * pldb + k_len_w) * ES);

    unsigned a_voff[T::A_LOADS], b_voff[T::B_LOADS];
    int a_kcol[T::A_LOADS], b_kcol[T::B_LOADS];
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
        const int c = (i * T::NW + wave) * 64 + lane;
        const int row = c / T::CA, lch = (c % T::CA) ^ T::a_key(row);
        a_kcol[i] = lch * (16 / ES);
        a_voff[i] = (unsigned)(row * plda * ES + lch * 16);
    }
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i) {
        const int c = (i * T::NW + wave) * 64 + lane;
        const int row = c / T::CB;
        if constexpr (T::BL == 0) {
            const int lbyte = ((c % T::CB) * 16) ^ T::b_key(row);
            const bool ok = n0 + lbyte / ES < pN;
            b_voff[i] = ok ? (unsigned)(row * pldb * ES + lbyte) : OOB_OFFSET;
            b_kcol[i] = 0;
        } else {
            const int lch = (c % T::CB) ^ T::a_key(row);      // same row bytes as A: same key
            b_kcol[i] = lch * (16 / ES);
            b_voff[i] = (unsigned)(row * pldb * ES + lch * 16);
        }
    }
    // Load instruction l of a slab request (A units first, then B units): asynchronous,
    // completion is counted by vmcnt.
#if defined(G355_DIAG_FILL_MODE) && G355_DIAG_FILL_MODE == 2
#define G355_FILL_BYTES 4      // timing-only: the same requests a quarter as wide
#else
#define G355_FILL_BYTES 16
#endif
#if defined(G355_DIAG_FILL_MODE) && G355_DIAG_FILL_MODE == 1
    // timing-only: the refill goes into registers that nothing reads (no LDS writes); they stay live until
    // the barrier the LDS data would have been needed at
    i32x4 diag_regs[T::A_LOADS + T::B_LOADS];
#endif
    // `mode` (a std::integral_constant): 0 default cache policy, 1 the B loads stream (one tile row), 2 the A loads
    // stream (one tile column).  A compile-time constant, chosen once outside the K loop: a run-time choice per
    // load would put every load into a basic block of its own and take the loop's schedule apart.
    // The streaming instantiation (a one-row grid: every byte of B is read once) over K-contiguous weights whose row
    // pitch is a power of two of 16 KiB or more (bf16 K = 8192, ...; from 8 KiB for the tiles of at most 32 rows)
    // walks the K range in a rotated order, workgroup tn starting tn slabs in.  The workgroups of such a grid advance
    // through K in step, and with such a pitch the rows of every workgroup's slab fall into the same few memory
    // channels at any one time (N = 28672, K = 8192 bf16: M = 16 83 us, 68 with the pitch padded by 256 bytes, 69
    // rotated; M = 64 104 -> 71, M = 256 139 -> 127).  Started at different slabs they spread over all channels.
    // Other pitches gain nothing (K = 28672: +-2 %; 8 KiB: fp8 K = 8192 at M = 16 39 -> 35 us with the small tiles,
    // +2-4 % with the taller ones), and row-major B loses 1-20 % (there the workgroups' simultaneous reads of
    // adjacent pieces of the same rows are what keeps DRAM pages open): both keep the plain order.  Only for whole
    // slabs (K range a multiple of BLOCK_K), so that no slab of the rotated order needs the test against the end of K.
    int rot = 0;
    auto issue_one = [&](auto mode, auto tail, int l, int slab, G355_LDS uint8_t *sbase) {
        constexpr int MODE = decltype(mode)::value;
        constexpr bool TAIL = decltype(tail)::value;     // false: the slab lies wholly inside the K range
        int kk = slab * BK;
        if constexpr (T::BL == 1 && MODE == 1) {
            // logical slab -> position in K; slabs requested past the last one stay outside the range
            int p = slab + rot;
            p = p >= kt_count ? p - kt_count : p;
            kk = (!TAIL || slab < kt_count) ? p * BK : kt_count * BK;
        }
        if (l < T::A_LOADS) {
            const int i = l, u = i * T::NW + wave;
            if (T::A_UNITS % T::NW == 0 || u < T::A_UNITS) {
                const unsigned off = (!TAIL || a_kcol[i] + kk < k_len) ? a_voff[i] + (unsigned)(kk * ES) : OOB_OFFSET;
#if defined(G355_DIAG_FILL_MODE) && G355_DIAG_FILL_MODE == 1
                diag_regs[l] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsA, off, 0, 0));
                return;
#endif
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (G355_LDS void *)(sbase + u * 1024), G355_FILL_BYTES, off, 0, 0,
                                                         MODE == 2 ? G355_LOAD_STREAM : G355_LOAD_DEFAULT);
            }
        } else {
            const int i = l - T::A_LOADS, u = i * T::NW + wave;
            if (T::B_UNITS % T::NW == 0 || u < T::B_UNITS) {
                unsigned off;
                if constexpr (T::BL == 0)
                    off = b_voff[i] + (unsigned)kk * (unsigned)(pldb * ES);
                else
                    off = (!TAIL || b_kcol[i] + kk < k_len) ? b_voff[i] + (unsigned)(kk * ES) : OOB_OFFSET;
#if defined(G355_DIAG_FILL_MODE) && G355_DIAG_FILL_MODE == 1
                diag_regs[l] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsB, off, 0, 0));
                return;
#endif
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB, (G355_LDS void *)(sbase + T::A_BYTES + u * 1024), G355_FILL_BYTES, off,
                                                         0, 0, MODE == 1 ? G355_LOAD_STREAM : G355_LOAD_DEFAULT);
            }
        }
    };
    constexpr int NL = T::A_LOADS + T::B_LOADS;   // load instructions per wave and slab

    // Ragged instantiation: the same requests into registers (`fetch`), elements of a K-contiguous operand
    // beyond the end of the K range cleared there, then written to the lane's LDS slot (`commit`).
    i32x4 staged[T::RG ? NL : 1];
    auto trim = [&](i32x4 v, int valid) {          // keep the first `valid` (< EPC) elements of a chunk
        constexpr int EPD = 4 / ES;                // elements per dword
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int keep = valid - d * EPD;
            const unsigned mask = keep >= EPD ? 0xffffffffu : keep <= 0 ? 0u : ((1u << (keep * 8 * ES)) - 1u);
            v[d] = (int)((unsigned)v[d] & mask);
        }
        return v;
    };
    auto fetch = [&](int slab) {
        const int kk = slab * BK;
#pragma unroll
        for (int l = 0; l < NL; ++l) {
            if (l < T::A_LOADS) {
                const int i = l, u = i * T::NW + wave;
                if (T::A_UNITS % T::NW == 0 || u < T::A_UNITS) {
                    const int valid = k_len - (a_kcol[i] + kk);
                    const unsigned off = (valid > 0) ? a_voff[i] + (unsigned)(kk * ES) : OOB_OFFSET;
                    i32x4 v = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsA, off, 0, 0));
                    staged[T::RG ? l : 0] = (valid < EPC) ? trim(v, valid) : v;
                }
            } else {
                const int i = l - T::A_LOADS, u = i * T::NW + wave;
                if (T::B_UNITS % T::NW == 0 || u < T::B_UNITS) {
                    if constexpr (T::BL == 0) {
                        // rows beyond the K range lie beyond the window; columns beyond N only feed outputs that are not stored
                        const unsigned off = b_voff[i] + (unsigned)kk * (unsigned)(pldb * ES);
                        staged[T::RG ? l : 0] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsB, off, 0, 0));
                    } else {
                        const int valid = k_len - (b_kcol[i] + kk);
                        const unsigned off = (valid > 0) ? b_voff[i] + (unsigned)(kk * ES) : OOB_OFFSET;
                        i32x4 v = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsB, off, 0, 0));
                        staged[T::RG ? l : 0] = (valid < EPC) ? trim(v, valid) : v;
                    }
                }
            }
        }
    };
    auto commit = [&](G355_LDS uint8_t *sbase) {
#pragma unroll
        for (int l = 0; l < NL; ++l) {
            const bool is_a = l < T::A_LOADS;
            const int i = is_a ? l : l - T::A_LOADS, u = i * T::NW + wave;
            if (is_a ? (T::A_UNITS % T::NW == 0 || u < T::A_UNITS) : (T::B_UNITS % T::NW == 0 || u < T::B_UNITS))
                *(G355_LDS i32x4 *)(sbase + (is_a ? 0 : T::A_BYTES) + u * 1024 + lane * 16) = staged[T::RG ? l : 0];
        }
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
    const int bk_row = wn * T::WTN + (lane % MI);   // K-contiguous B: the lane's n row, k group a_kg

    typedef typename std::conditional<MI == 32, f32x16, f32x4>::type acc_t;
    acc_t acc[T::TN][T::TM];
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
        for (int i = 0; i < T::TM; ++i)
#pragma unroll
            for (int r = 0; r < T::ACC; ++r)
                acc[j][i][r] = 0.f;

    // Fragments of one MFMA k-step, double buffered in registers: while the MFMAs of k-step s
    // run, the LDS reads of k-step s+1 are in flight.
    typedef typename std::conditional<ES == 2, bf16x8, i32x8>::type frag_t;
    frag_t af[2][T::TM], bfr[2][T::TN];

    // Fragment `u` of k-step `kstep` of LDS stage `stage` into register buffer `buf`:
    // u < TM is the A fragment of MFMA tile row u, otherwise the B fragment of tile column u-TM.
    // (`dslot` >= 0: a B fragment goes to slot dslot of the flat B register array instead of [buf][j]: K-loop form 6)
    auto load_frag = [&](const G355_LDS uint8_t *sA, int kstep, int buf, int u, int dslot = -1) {
        const G355_LDS uint8_t *sB = sA + T::A_BYTES;
        const int k0 = kstep * T::KI;
        if (u < T::TM) {
            const int i = u;
            if constexpr (ES == 2) {
                const int chunk = (k0 + a_kg * T::KL) / 8;
                af[buf][i] = *(const G355_LDS bf16x8 *)(sA + T::a_off(a_row + i * MI, chunk));
            } else {
                const int chunk = (k0 + a_kg * T::KL) / 16;
                i32x4 lo = *(const G355_LDS i32x4 *)(sA + T::a_off(a_row + i * MI, chunk));
                i32x4 hi = *(const G355_LDS i32x4 *)(sA + T::a_off(a_row + i * MI, chunk + 1));
                af[buf][i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        } else {
            const int j = u - T::TM;
            frag_t &dst = dslot < 0 ? bfr[buf][j] : bfr[dslot / T::TN][dslot % T::TN];
            if constexpr (T::BL == 1 && ES == 2) {
                const int chunk = (k0 + a_kg * T::KL) / 8;
                dst = *(const G355_LDS bf16x8 *)(sB + T::a_off(bk_row + j * MI, chunk));
            } else if constexpr (T::BL == 1) {
                const int chunk = (k0 + a_kg * T::KL) / 16;
                i32x4 lo = *(const G355_LDS i32x4 *)(sB + T::a_off(bk_row + j * MI, chunk));
                i32x4 hi = *(const G355_LDS i32x4 *)(sB + T::a_off(bk_row + j * MI, chunk + 1));
                dst = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            } else if constexpr (ES == 2) {
                short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (G355_LDS short4_t *)(sB + T::b_off(k0 + b_krow_l, (b_ncol + j * MI) * 2)));
                short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (G355_LDS short4_t *)(sB + T::b_off(k0 + b_krow_l + TRK, (b_ncol + j * MI) * 2)));
                typedef short short8_t __attribute__((ext_vector_type(8)));
                short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                dst = __builtin_bit_cast(bf16x8, v);
            } else {
                int2_t q[4];
#pragma unroll
                for (int h = 0; h < 4; ++h)
                    q[h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                        (G355_LDS int2_t *)(sB + T::b_off(k0 + b_krow_l + h * TRK, b_ncol + j * MI)));
                i32x4 lo = __builtin_shufflevector(q[0], q[1], 0, 1, 2, 3);
                i32x4 hi = __builtin_shufflevector(q[2], q[3], 0, 1, 2, 3);
                dst = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    constexpr int NF = T::TM + T::TN;     // fragments per k-step
    // acc[j][i] += B fragment in flat slot `bslot` x A fragment af[abuf][i]
    auto mma_ops = [&](int bslot, int abuf, int j, int i) {
        const frag_t &bf_ = bfr[bslot / T::TN][bslot % T::TN];
        const frag_t &af_ = af[abuf][i];
        if constexpr (ES == 2 && T::FT == 1 && MI == 32)
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, bf_),
                                                               __builtin_bit_cast(f16x8, af_), acc[j][i], 0, 0, 0);
        else if constexpr (ES == 2 && T::FT == 1)
            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, bf_),
                                                               __builtin_bit_cast(f16x8, af_), acc[j][i], 0, 0, 0);
        else if constexpr (ES == 2 && MI == 32)
            acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf_, af_, acc[j][i], 0, 0, 0);
        else if constexpr (ES == 2)
            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf_, af_, acc[j][i], 0, 0, 0);
        else if constexpr (MI == 32)
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bf_, af_, acc[j][i], 0, 0, 0, 0, 0, 0);
        else
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf_, af_, acc[j][i], 0, 0, 0, 0, 0, 0);
    };
    auto mma_one = [&](int buf, int j, int i) { mma_ops(buf * T::TN + j, buf, j, i); };

    // ---- pipeline: prologue, main K loop, epilogue (Algorithm 8's three phases) ----
    // Ring of NS LDS stages; slab kt lives in stage kt % NS.  One barrier per slab, placed
    // before the last k-step's MFMAs (whose fragments are already in registers).  It certifies
    // two things at once: every wave has finished reading the current stage, and every wave's
    // loads of slab kt+1 have landed (a wave waits for all but its newest NS-2 slab requests
    // first).  Right after it the freed stage is refilled with slab kt+NS -- a request has NS-1
    // whole iterations to land -- and the first fragments of the next stage are fetched under
    // the last k-step's MFMAs.  Requests past the last slab are out-of-window loads: they move
    // no data and keep the loop body branch-free.
    static_assert(T::KSTEPS % 2 == 0, "fragment double buffering needs an even number of k-steps");
    // vmcnt allowance at the barrier of iteration kt: slabs kt+2 .. kt+NS-1 may still be in
    // flight.  Only instructions that every wave issues are counted (ragged unit counts), so a
    // wave never waits for less than it must.
    constexpr int FULL = T::common_loads();
    constexpr int ALLOW = (T::NS - 2) * FULL;
    static_assert((T::NS - 1) * FULL <= 63, "vmcnt is a 6-bit counter");
    constexpr int LF = T::LF;
    // form 3: LDS read instructions per k-step and how they are spread over its MN MFMAs
    constexpr int MN = T::TM * T::TN;
#ifndef G355_LF5_SPREAD4
#define G355_LF5_SPREAD4 2      // quarters of a k-step's MFMAs over which the next fragments' reads are spread
#endif
    constexpr int H5 = MN * G355_LF5_SPREAD4 / 4 > 0 ? MN * G355_LF5_SPREAD4 / 4 : 1;   // form 5: MFMAs of a k-step that carry the next k-step's fragment reads
    constexpr int NFR = T::TM * (ES == 2 ? 1 : 2) + T::TN * (T::BL == 1 ? (ES == 2 ? 1 : 2) : (ES == 2 ? 2 : 4));
    constexpr int RD_A = (NFR + (MN > 1 ? MN / 2 : 1) - 1) / (MN > 1 ? MN / 2 : 1);
    constexpr int RD_PAIRS = NFR / RD_A, RD_REM = NFR - RD_PAIRS * RD_A;
    auto publish = [&]() {
#if defined(G355_DIAG_FILL_MODE) && G355_DIAG_FILL_MODE == 1
#pragma unroll
        for (int l = 0; l < NL; ++l)
            asm volatile("" ::"v"(diag_regs[l]));
#endif
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(ALLOW) : "memory");
    };

    // The compiler cannot tell which LDS bytes a direct-to-LDS load will write, and before an LDS
    // read that might touch them it waits for every such load in flight (vmcnt(0)), which would
    // serialise each refill with the reads that follow it.  The part of an iteration between two
    // barriers therefore lives in a function whose two stage pointers are `__restrict__`: it
    // refills only the stage that was just freed and reads only the next one, the two never
    // overlap, and the waits that order refills against reads are the explicit ones of publish().
    G355_LDS uint8_t *const lds = (G355_LDS uint8_t *)smem;
    auto mma_kstep = [&](int buf) __attribute__((always_inline)) {
#ifndef G355_DIAG_SKIP_MFMA
#pragma unroll
        for (int m = 0; m < T::TM * T::TN; ++m)
            mma_one(buf, m / T::TM, m % T::TM);
#else
        (void)buf;
#endif
    };
    // k-steps 0 .. KSTEPS-2 of the slab in `cur` (its first fragments are in registers), then the
    // slab's barrier
    auto until_barrier = [&](const G355_LDS uint8_t *cur) __attribute__((always_inline)) {
#pragma unroll
        for (int kstep = 0; kstep < T::KSTEPS - 1; ++kstep) {
            if constexpr (LF == 5) {
                // form 5: the order is written out -- MFMA m of the k-step is preceded by its share of the next
                // k-step's fragment reads (spread over the first half of the MFMAs), and nothing may move
                // across the fence after it
#pragma unroll
                for (int m = 0; m < MN; ++m) {
                    // fragments u with floor(u * H5 / NF) == m
#pragma unroll
                    for (int u = (m * NF + H5 - 1) / H5; u < ((m + 1) * NF + H5 - 1) / H5 && u < NF; ++u)
                        load_frag(cur, kstep + 1, (kstep + 1) & 1, u);
                    mma_one(kstep & 1, m / T::TM, m % T::TM);
                    G355_LF5_FENCE(m);
                }
                continue;
            }
#ifndef G355_DIAG_SKIP_FRAG
#pragma unroll
            for (int u = 0; u < NF; ++u)
                load_frag(cur, kstep + 1, (kstep + 1) & 1, u);
#endif
            mma_kstep(kstep & 1);
            if constexpr (LF == 3 || LF == 4) {
                sched_reads_then_mfma<RD_PAIRS, RD_A>();
                if constexpr (RD_REM > 0) {
                    __builtin_amdgcn_sched_group_barrier(0x100, RD_REM, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                }
                if constexpr (MN - RD_PAIRS - (RD_REM > 0) > 0)
                    __builtin_amdgcn_sched_group_barrier(0x008, MN - RD_PAIRS - (RD_REM > 0), 0);
            }
        }
        publish();
    };
    // from the barrier of slab kt to the barrier of slab kt + 1
    auto after_barrier = [&](auto mode, auto tail, G355_LDS uint8_t *__restrict__ freed, const G355_LDS uint8_t *__restrict__ next, int kt)
                             __attribute__((always_inline)) {
        if constexpr (LF == 5) {
            // form 5: refill loads one every MN / NL MFMAs, the next slab's first fragments over the first half
#pragma unroll
            for (int m = 0; m < MN; ++m) {
                // loads l with floor(l * MN / NL) == m, fragments u with floor(u * H5 / NF) == m
#pragma unroll
                for (int l = (m * NL + MN - 1) / MN; l < ((m + 1) * NL + MN - 1) / MN && l < NL; ++l)
                    issue_one(mode, tail, l, kt + T::NS, freed);
#pragma unroll
                for (int u = (m * NF + H5 - 1) / H5; u < ((m + 1) * NF + H5 - 1) / H5 && u < NF; ++u)
                    load_frag(next, 0, 0, u);
                mma_one((T::KSTEPS - 1) & 1, m / T::TM, m % T::TM);
                G355_LF5_FENCE(m);
            }
            until_barrier(next);
            return;
        }
#ifndef G355_DIAG_SKIP_FILL
#pragma unroll
        for (int l = 0; l < NL; ++l)
            issue_one(mode, tail, l, kt + T::NS, freed);
#endif
        // form 2: no memory instruction may be scheduled across this point (ALU and MFMA
        // instructions may), or the refill drifts down the iteration it has to land in
        if constexpr (LF == 2)
            __builtin_amdgcn_sched_barrier(0xF);
#ifndef G355_DIAG_SKIP_FRAG
#pragma unroll
        for (int u = 0; u < NF; ++u)
            load_frag(next, 0, 0, u);
#endif
        mma_kstep((T::KSTEPS - 1) & 1);
        if constexpr (LF == 4)
            sched_spread_fills<0, MN, NL, NFR>();
        if constexpr (LF == 3) {
            // the refill two loads per MFMA, then the fragment reads as in the other k-steps
            constexpr int FP = (NL + 1) / 2 < MN / 2 ? (NL + 1) / 2 : MN / 2;     // MFMAs that carry fills
            constexpr int RP = MN - FP;                                            // MFMAs left for the reads
            constexpr int A3 = (NFR + (RP > 1 ? RP - 1 : 1) - 1) / (RP > 1 ? RP - 1 : 1);
            constexpr int P3 = NFR / A3, R3 = NFR - P3 * A3;
            if constexpr (FP > 0) {
                sched_fills_then_mfma<FP - 1, 2>();
                __builtin_amdgcn_sched_group_barrier(0x020, NL - 2 * (FP - 1), 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            } else {
                __builtin_amdgcn_sched_group_barrier(0x020, NL, 0);
            }
            sched_reads_then_mfma<P3, A3>();
            if constexpr (R3 > 0) {
                __builtin_amdgcn_sched_group_barrier(0x100, R3, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            if constexpr (RP - P3 - (R3 > 0) > 0)
                __builtin_amdgcn_sched_group_barrier(0x008, RP - P3 - (R3 > 0), 0);
        }
        if (LF != 0 || kt + 1 < kt_count)
            until_barrier(next);
    };

    if constexpr (T::RG) {
        if (kt_count > 0) {
            fetch(0);
            commit(lds);
            __syncthreads();
            for (int kt = 0; kt < kt_count; ++kt) {
                const G355_LDS uint8_t *cur = lds + (kt & 1) * T::STAGE;
                if (kt + 1 < kt_count)
                    fetch(kt + 1);                   // in flight during this slab's MFMAs
#pragma unroll
                for (int u = 0; u < NF; ++u)
                    load_frag(cur, 0, 0, u);
#pragma unroll
                for (int kstep = 0; kstep < T::KSTEPS; ++kstep) {
                    if (kstep + 1 < T::KSTEPS) {
#pragma unroll
                        for (int u = 0; u < NF; ++u)
                            load_frag(cur, kstep + 1, (kstep + 1) & 1, u);
                    }
                    mma_kstep(kstep & 1);
                }
                // the other stage was last read in the previous iteration, which every wave has left
                if (kt + 1 < kt_count)
                    commit(lds + ((kt + 1) & 1) * T::STAGE);
                __syncthreads();
            }
        }
    } else if (kt_count > 0) {
      auto pipeline = [&](auto mode) __attribute__((always_inline)) {
        if constexpr (T::BL == 1 && decltype(mode)::value == 1) {
            const unsigned pitch = (unsigned)pldb * ES;
            constexpr unsigned MIN_PITCH = BM <= 32 ? 8192 : 16384;
            rot = (k_len % BK == 0 && pitch >= MIN_PITCH && (pitch & (pitch - 1)) == 0) ? tn % kt_count : 0;
        }
#pragma unroll
        for (int s = 0; s < T::NS; ++s)
#pragma unroll
            for (int l = 0; l < NL; ++l)
                issue_one(mode, std::true_type{}, l, s, lds + s * T::STAGE);
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((T::NS - 1) * FULL) : "memory");
        if constexpr (LF == 6) {
            // Form 6: B fragments are not double-buffered per k-step but pass through a ring of R6 register
            // slots, each read D6 blocks ahead of its use (a block = the TM MFMAs that share one B fragment; a
            // slab has NB of them).  Only the A fragments keep two buffers.  That is 16 (2x4 wave grid) or 48 (4x2) fewer registers in
            // the 256x256x64 eight-wave tiles, whose loop then fits without the compiler folding the buffers together.
            // The current stage is read until block NB-1-D6 has issued its prefetch, so the slab's barrier sits
            // there; the refill and the next slab's first fragments go out in the D6 blocks after it.
            constexpr int NB = T::KSTEPS * T::TN, D6 = 3, R6 = 4, TM_ = T::TM, TN_ = T::TN;
            static_assert(TN_ >= D6 && NB % R6 == 0 && 2 * TN_ >= R6 && T::KSTEPS >= 2, "tile does not fit K-loop form 6");
            auto mfmas = [&](int f) __attribute__((always_inline)) {
#pragma unroll
                for (int i = 0; i < TM_; ++i)
                    mma_ops(f % R6, (f / TN_) & 1, f % TN_, i);
            };
            // blocks 0 .. NB-D6-1 of the slab in `st`, then its barrier
            auto head = [&](const G355_LDS uint8_t *st) __attribute__((always_inline)) {
#pragma unroll
                for (int f = 0; f < NB - D6; ++f) {
                    const int g = f + D6, kstep = f / TN_, j = f % TN_;
                    load_frag(st, g / TN_, 0, TM_ + g % TN_, g % R6);
                    if (kstep + 1 < T::KSTEPS) {
#pragma unroll
                        for (int i = (j * TM_ + TN_ - 1) / TN_; i < ((j + 1) * TM_ + TN_ - 1) / TN_ && i < TM_; ++i)
                            load_frag(st, kstep + 1, (kstep + 1) & 1, i);
                    }
                    mfmas(f);
                    __builtin_amdgcn_sched_barrier(0);
                }
                publish();
            };
            // from the barrier of slab kt to the barrier of slab kt + 1
            auto span = [&](auto tail, G355_LDS uint8_t *__restrict__ freed, const G355_LDS uint8_t *__restrict__ next, int kt)
                            __attribute__((always_inline)) {
#pragma unroll
                for (int t = 0; t < D6; ++t) {
                    const int f = NB - D6 + t;
#pragma unroll
                    for (int l = (t * NL + D6 - 1) / D6; l < ((t + 1) * NL + D6 - 1) / D6 && l < NL; ++l)
                        issue_one(mode, tail, l, kt + T::NS, freed);
                    load_frag(next, 0, 0, TM_ + t, (f + D6) % R6);
#pragma unroll
                    for (int i = (t * TM_ + D6 - 1) / D6; i < ((t + 1) * TM_ + D6 - 1) / D6 && i < TM_; ++i)
                        load_frag(next, 0, 0, i);
                    mfmas(f);
                    __builtin_amdgcn_sched_barrier(0);
                }
                head(next);
            };
#pragma unroll
            for (int i = 0; i < TM_; ++i)
                load_frag(lds, 0, 0, i);
#pragma unroll
            for (int g = 0; g < D6; ++g)
                load_frag(lds, 0, 0, TM_ + g, g % R6);
            head(lds);
            int stage6 = 0, kt6 = 0;
            const int end6 = kt_count - 1;
            int main6 = k_len / BK - T::NS;
            main6 = main6 < end6 ? main6 : end6;
            for (; kt6 < main6; ++kt6) {
                const int next = (stage6 + 1 == T::NS) ? 0 : stage6 + 1;
                span(std::false_type{}, lds + stage6 * T::STAGE, lds + next * T::STAGE, kt6);
                stage6 = next;
            }
            for (; kt6 < end6; ++kt6) {
                const int next = (stage6 + 1 == T::NS) ? 0 : stage6 + 1;
                span(std::true_type{}, lds + stage6 * T::STAGE, lds + next * T::STAGE, kt6);
                stage6 = next;
            }
#pragma unroll
            for (int f = NB - D6; f < NB; ++f)
                mfmas(f);
            return;
        }
#pragma unroll
        for (int u = 0; u < NF; ++u)
            load_frag(lds, 0, 0, u);
#ifdef G355_DIAG_SKIP_FRAG
#pragma unroll
        for (int u = 0; u < NF; ++u)
            load_frag(lds, 1, 1, u);      // both register buffers hold real fragments of the first slab
#endif
        until_barrier(lds);
        int stage = 0;                         // stage of slab kt
        // forms 1 and 2 peel the last slab off (see Tile)
        const int kt_end = kt_count - (LF != 0);
        int kt = 0;
        // Iterations whose refill (slab kt + NS) lies wholly inside the K range run a copy of the loop without the
        // per-chunk test against the end of K (three vector ALU instructions and a register per load of a
        // K-contiguous operand; with them the 256x256 tiles on K-contiguous B spilled); the last NS + 1 do test.
        int kt_main = k_len / BK - T::NS;
        kt_main = kt_main < kt_end ? kt_main : kt_end;
        for (; kt < kt_main; ++kt) {
            const int next = (stage + 1 == T::NS) ? 0 : stage + 1;
            after_barrier(mode, std::false_type{}, lds + stage * T::STAGE, lds + next * T::STAGE, kt);
            stage = next;
        }
        for (; kt < kt_end; ++kt) {
            const int next = (stage + 1 == T::NS) ? 0 : stage + 1;
            after_barrier(mode, std::true_type{}, lds + stage * T::STAGE, lds + next * T::STAGE, kt);
            stage = next;
        }
        if constexpr (LF != 0)
            mma_kstep((T::KSTEPS - 1) & 1);
      };
      // the streaming instantiation: B is read once and streams (see Tile::STREAMABLE_B); a kernel has one copy of the loop
      if constexpr (T::STREAMABLE_B) {
          pipeline(std::integral_constant<int, 1>{});
      } else if constexpr (T::STREAMABLE_A) {
          if (stream_a)
              pipeline(std::integral_constant<int, 2>{});
          else
              pipeline(std::integral_constant<int, 0>{});
      } else {
          pipeline(std::integral_constant<int, 0>{});
      }
    }
    // nothing may still be in flight towards LDS when the workgroup ends
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue: a lane holds, per MFMA tile, output row m = lane % MI and columns
    //      n = 8*(r/4) + 4*(lane/32) + r%4 (32x32) or n = 4*(lane/16) + r (16x16).  Stored from
    //      there, one instruction would write 16- or 32-byte pieces of many rows; instead every
    //      wave passes its accumulators through a private piece of the (now free) LDS ring, one
    //      MFMA row block (MI rows of its wave tile) at a time, and stores whole row segments of
    //      its tile: 128 bytes and more per row.  Staged rows are padded by 16 bytes so that the
    //      16-byte writes of a column of lanes spread over the banks. ----
    typedef typename std::conditional<T::FT == 1, _Float16, __bf16>::type out_t;
    typedef typename std::conditional<T::FT == 1, f16x8, bf16x8>::type out8_t;
    constexpr int ST_ROW = T::WTN * 4 + 16;                 // bytes per staged row
    constexpr int ST_CPR = T::WTN / 8;                      // 8-float chunks per row
    static_assert(T::NW * MI * ST_ROW <= T::NS * T::STAGE, "the staging rows of all waves must fit the LDS ring");
    const float alpha = args.alpha, beta = args.beta;
    // every wave's requests towards LDS have landed (above) and every wave is past its last fragment read
    __syncthreads();
    G355_LDS uint8_t *stg = lds + wave * (MI * ST_ROW);
    const int st_w = (lane % MI) * ST_ROW + 16 * (lane / MI);      // this lane's row and 4-column group
    const int row0 = m0 + wm * T::WTM, col0 = n0 + wn * T::WTN;    // origin of the wave tile
#pragma unroll
    for (int i = 0; i < T::TM; ++i) {
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int q = 0; q < T::ACC / 4; ++q) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = acc[j][i][q * 4 + r];
                *(G355_LDS f32x4 *)(stg + st_w + (j * MI + q * 8) * 4) = v;
            }
        // the wave reads back what it wrote itself (LDS operations of one wave complete in order):
        // 8 consecutive columns per lane, so that a 16-bit result leaves as one 16-byte store
#pragma unroll
        for (int c0 = 0; c0 < MI * ST_CPR; c0 += 64) {
            const int c = c0 + lane;
            const int m = row0 + i * MI + c / ST_CPR, n = col0 + (c % ST_CPR) * 8;
            if ((MI * ST_CPR % 64 != 0 && c >= MI * ST_CPR) || m >= pM || n >= pN)
                continue;
            const G355_LDS uint8_t *src = stg + (c / ST_CPR) * ST_ROW + (c % ST_CPR) * 32;
            const f32x4 lo = *(const G355_LDS f32x4 *)src, hi = *(const G355_LDS f32x4 *)(src + 16);
            if (out_mode != 0) {
                // split-K slabs have rows of N rounded up to 8 floats (whole 32-byte stores also at a ragged edge)
                const size_t nw = T::RG ? (size_t)(pN + 7) / 8 * 8 : (size_t)pN;   // (N is a multiple of 8 otherwise)
                float *dst = (out_mode == 1)
                                 ? args.ws + ((bz * args.split_k + ks) * pM + m) * nw + n
                                 : args.ws + ((size_t)(2 * blockIdx.x + seg) * BM + (m - m0)) * BN + (n - n0);
                *(f32x4 *)dst = lo;
                *(f32x4 *)(dst + 4) = hi;
            } else {
                out_t *dst = (out_t *)pC + bz * args.stride_c + (size_t)m * pldc + n;
                out8_t o;
                if (beta != 0.f) {
                    const out8_t cin = *(const out8_t *)dst;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        o[r] = (out_t)__builtin_fmaf(beta, (float)cin[r], lo[r] * alpha);
                        o[r + 4] = (out_t)__builtin_fmaf(beta, (float)cin[r + 4], hi[r] * alpha);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        o[r] = (out_t)(lo[r] * alpha);
                        o[r + 4] = (out_t)(hi[r] * alpha);
                    }
                }
                if (!T::RG || n + 8 <= pN) {
                    *(out8_t *)dst = o;
                } else {
                    // ragged edge of C: nothing beyond column N - 1 is written
#pragma unroll
                    for (int r = 0; r < 8; ++r)
                        if (n + r < pN)
                            dst[r] = o[r];
                }
            }
        }
    }
    }   // segments
}

}  // namespace g355
