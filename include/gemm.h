/*
 * gemm.h -- C ABI of the MI355X (gfx950) GEMM library.
 *
 * Computes C = alpha * A * B + beta * C (the paper's Section II-A definition; beta defaults to 0):
 *   A  M x K, row-major, leading dimension lda (elements), bf16, IEEE fp16 or fp8 e4m3 (OCP "e4m3fn")
 *   B  K x N, row-major, leading dimension ldb (GEMM_B_ROW_MAJOR, the default), or stored as its
 *      transpose, N x K row-major, K-contiguous, ldb >= K (GEMM_B_K_CONTIGUOUS: the operand layout of
 *      the paper's own runs, Section V, and of an nn.Linear weight)
 *   C  M x N, row-major, leading dimension ldc, bf16 (fp16 for fp16 inputs), rounded to nearest
 *      even from an fp32 accumulator.
 * One launch computes one product, a strided batch of equal shapes, or a group of different shapes.
 * A, B, C, the split-K / Stream-K workspace and a grouped launch's table are DEVICE memory owned by the caller; the library
 * never allocates, frees or copies them.  Per-tensor fp8 scales enter as
 * cfg.alpha = scale_a * scale_b.
 *
 * The kernel that runs is picked by gemm_select(): a deterministic analytical model of
 * the tiling hierarchy (Section IV of the paper: Algorithms 3-9) evaluated for every
 * compiled kernel variant -- no timing, no GPU call, no allocation.
 *
 * All functions return 0 on success or a negative gemm_status; nothing is launched when
 * an error is returned.  No function throws or aborts.
 */
#ifndef GEMM355_GEMM_H
#define GEMM355_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GEMM_ABI_VERSION 8u

typedef enum gemm_dtype {
    GEMM_BF16 = 0,     /* A, B bf16; C bf16 */
    GEMM_FP8_E4M3 = 1, /* A, B one byte per element, OCP e4m3fn (max finite 448); C bf16 */
    GEMM_FP16 = 2      /* A, B IEEE binary16 (the precision of the paper's runs, Section V); C binary16.
                          Same tile list, calibration constants and model row as bf16. */
} gemm_dtype;

typedef enum gemm_b_layout {
    GEMM_B_ROW_MAJOR = 0,    /* B[k][n] at B + k*ldb + n */
    GEMM_B_K_CONTIGUOUS = 1  /* B[k][n] at B + n*ldb + k */
} gemm_b_layout;

typedef enum gemm_status {
    GEMM_OK = 0,
    GEMM_ERR_NULL = -1,        /* a required pointer is NULL */
    GEMM_ERR_SHAPE = -2,       /* M, N or K < 1, or beyond the 32-bit tile arithmetic */
    GEMM_ERR_DTYPE = -3,       /* dtype is not a gemm_dtype */
    GEMM_ERR_CFG_ILLEGAL = -4, /* cfg fields do not describe a compiled kernel legal for the shape */
    GEMM_ERR_ALIGN = -5,       /* a pointer, leading dimension or batch stride is not a multiple of 16 bytes */
    GEMM_ERR_WORKSPACE = -6,   /* split_k > 1 and the registered workspace is missing or too small */
    GEMM_ERR_ABI = -7,         /* cfg.abi_version differs from GEMM_ABI_VERSION */
    GEMM_ERR_HIP = -8,         /* the HIP runtime refused the launch */
    GEMM_ERR_INDEX = -9        /* gemm_cfg_at: index outside [0, gemm_cfg_count) */
} gemm_status;

/* Bottleneck label of a prediction (Section IV-D's taxonomy). */
typedef enum gemm_bottleneck {
    GEMM_BOUND_COMPUTE_FULL = 0, /* all CUs busy, matrix cores limit */
    GEMM_BOUND_COMPUTE_UNDER = 1,/* matrix cores limit, but fewer tiles than CUs in the last wave */
    GEMM_BOUND_LS_ISSUE = 2,     /* per-CU vector-memory issue rate */
    GEMM_BOUND_LDS = 3,          /* LDS read bandwidth */
    GEMM_BOUND_L2 = 4,           /* L2 bandwidth */
    GEMM_BOUND_MALL = 5,         /* Infinity Cache (MALL) bandwidth */
    GEMM_BOUND_HBM = 6,          /* HBM bandwidth + latency */
    GEMM_BOUND_LAUNCH = 7        /* fixed launch / prologue / epilogue cost dominates */
} gemm_bottleneck;

/*
 * Hardware descriptor H of the model (Section IV: CU count, cache scopes, bandwidths,
 * memory latency, matrix-instruction issue intervals).  Bandwidths are bytes per
 * compute clock; the defaults describe one MI355X and are compiled in.
 */
typedef struct gemm_hw {
    int32_t n_cu;              /* compute units on the device (256) */
    int32_t n_xcd;             /* L2 scopes; CUs per L2 = n_cu / n_xcd (8 -> 32) */
    int32_t simd_per_cu;       /* 4 */
    int32_t reserved0;
    double lds_bytes;          /* per CU (163840) */
    double l2_bytes;           /* per XCD (4 MiB) */
    double mall_bytes;         /* device (256 MiB) */
    double clk_ghz;            /* sustained compute clock used to convert clocks to time */
    double hbm_bytes_per_clk;  /* device total */
    double mall_bytes_per_clk; /* device total */
    double l2_bytes_per_clk;   /* per XCD */
    double lds_bytes_per_clk;  /* per CU, ds_read_b128 fragment reads */
    double lds_tr_bytes_per_clk; /* per CU, transpose fragment reads (ds_read_b64_tr_*) */
    double vmem_bytes_per_clk; /* per CU vector-memory (L1) rate */
    double mem_latency_clk;    /* L_lat of Algorithm 7 */
    double cache_eff_frac;     /* fraction of a cache's capacity that holds reusable tiles */
    double launch_clk;         /* fixed cost per kernel launch, clocks */
    double wg_overhead_clk;    /* fixed cost per workgroup (dispatch, address setup, drain) */
    double epilogue_clk;       /* fixed part of a tile's store stage */
    double reduce_launch_clk;  /* fixed cost of the split-K reduction pass */
    double under_occ_frac;     /* slab cost of a tile that has a CU to itself, as a fraction of its cost when the CU is full */
    double seg_eff_lo;         /* share of the HBM rate reached with 32-byte row segments (1 from 256 bytes up) */
    double overlap_frac;       /* with two or more workgroups resident per CU: share of a tile's prologue and store stage
                                  that hides under the other workgroups' K loops in every wave but the last (0 .. 1) */
    double l_mi_clk[2][2];     /* issue interval L_MI of one MFMA on workload-like operands (the chip is power-limited):
                                  [0: 16-bit, 1: fp8][0: 32x32, 1: 16x16], in clk_ghz clocks */
    double fill_issue_bytes_per_clk; /* bytes of a slab's direct-to-LDS fill the waves of a CU issue per clock, taken
                                  out of their MFMA streams (added to Algorithm 3's latency, not overlapped) */
    double slab_sync_clk;      /* barrier and first-fragment wait of one K slab, clocks */
} gemm_hw;

/*
 * A kernel configuration: plain data, no hidden pointers, so it can be copied and cached.
 * gemm_select / gemm_cfg_at fill every field; gemm_run validates them again.
 */
typedef struct gemm_cfg {
    uint32_t abi_version;
    int32_t dtype;            /* gemm_dtype */
    int64_t M, N, K;
    int64_t lda, ldb, ldc;    /* elements; gemm_select sets K, N (K for K-contiguous B), N */
    int32_t kernel_id;        /* index into the compiled variant table */
    uint16_t block_m, block_n, block_k; /* workgroup tile M_T x N_T x K_T */
    uint8_t waves_m, waves_n; /* wave grid inside the workgroup */
    uint8_t mfma;             /* 32: 32x32xk MFMA, 16: 16x16xk MFMA */
    uint8_t k_unroll;         /* MFMA k-steps unrolled per K_T slab (block_k / MI_K) */
    uint16_t split_k;         /* spatial K unroll: K slices computed by different workgroups */
    uint16_t group_m;         /* cache-tile height in tiles (Algorithm 6's f_m); tiles run column-major inside a band of group_m tile rows */
    uint16_t group_n;         /* cache-tile width f_n = CUs per L2 / f_m (informational) */
    uint8_t xcd_remap;        /* 1: workgroup ids are renumbered so that each XCD owns a contiguous id range */
    uint8_t stages;           /* LDS ring depth: K_T slabs resident or in flight per workgroup */
    uint16_t reserved1;       /* 0 */
    uint8_t b_layout;         /* gemm_b_layout */
    uint8_t stream_k;         /* 1: the last partial wave of tiles is split along K over sk_workers workgroups (needs split_k = 1) */
    uint16_t sk_workers;      /* stream-K workgroups G (= workgroup slots of the device for this variant); 0 when stream_k = 0 */
    float alpha;              /* default 1; the caller may overwrite it before gemm_run */
    int32_t bottleneck;       /* gemm_bottleneck of the prediction */
    float beta;               /* default 0; C = alpha*A*B + beta*C (Section II-A).  0: C is written without being read */
    double predicted_us;      /* model's total latency for this cfg */
    int32_t batch;            /* independent problems of this shape in one launch (default 1) */
    int32_t groups;           /* 0, or the number of groups of a grouped cfg (gemm_select_grouped): M, N, K then hold
                                 the largest extents over the groups and the cfg runs through gemm_run_grouped only */
    int64_t stride_a, stride_b, stride_c; /* elements between consecutive problems' A, B, C; gemm_select_batched
                                             sets the dense values M*lda, (K or N)*ldb, M*ldc */
} gemm_cfg;

/* Terms of the model for one cfg (clocks unless said otherwise), for tests and reports. */
typedef struct gemm_prediction {
    double n_mi;          /* Algorithm 3: matrix instructions per workgroup tile and K slab */
    double l_mt_ideal;    /* Algorithm 3: L_MT = L_MI * N_MI, spread over the SIMDs the workgroup's waves occupy */
    double l_compute;     /* compute latency of one K step of the tiles resident on a CU: (L_MT + fill bytes /
                             fill_issue_bytes_per_clk + slab_sync_clk) per tile, times the resident tiles */
    double tiles;         /* Algorithm 4: output tiles x split_k */
    double waves;         /* Algorithm 4: omega */
    double active_cu;     /* Algorithm 4: CUs busy in the last wave */
    double f_m, f_n;      /* Algorithm 6 pair chosen for the L2 scope */
    double h_l2, h_mall;  /* Algorithm 5 hit rates after the capacity derate */
    double l_issue, l_lds, l_l2, l_mall, l_hbm; /* Algorithm 7 terms, full wave */
    double l_mem;         /* Algorithm 7: max of the terms above, full wave */
    double l_mem_tail;    /* same with C = active_cu */
    double l_prologue, l_epilogue, l_iter; /* Algorithm 8, full wave */
    double iters;         /* Algorithm 8: I */
    double l_tile;        /* Algorithm 8, full wave */
    double l_tile_tail;   /* Algorithm 8 with C = active_cu */
    double l_reduce;      /* split-K reduction pass, clocks (0 when split_k = 1) */
    double l_total;       /* Algorithm 9 with the tail reading, clocks */
    double total_us;
    int32_t bottleneck;
    int32_t occupancy;    /* workgroups of the variant the model takes to be resident on one CU (slots per CU in Algorithm 4) */
} gemm_prediction;

uint32_t gemm_abi_version(void);
const char *gemm_strerror(int status);

/*
 * Analytical selection (Algorithms 3-9 over every compiled variant, arg-min of predicted
 * latency, deterministic tie-break).  Pure host code: works with no GPU present.
 * out: caller-owned.  Total on M, N, K >= 1 (up to 2^30 each).  The cfg's leading dimensions are set to the
 * smallest legal ones: K, N (K for K-contiguous B) and N, each rounded up to a whole number of 16-byte
 * chunks (8 16-bit or 16 fp8 elements; ldc: 8 elements); the caller may overwrite them with larger
 * multiples of that.  N and K themselves need not be such multiples: gemm_run then runs the variant's
 * instantiation that trims the ragged ends in registers (slower than the direct-to-LDS one; the model
 * does not price the difference).  A grid of one tile row (M <= BLOCK_M) over weights larger than the hardware
 * descriptor's mall_bytes runs the variant's weight-streaming instantiation: B's loads carry the non-temporal hint,
 * and K-contiguous weights whose row pitch is a power of two of 16 KiB or more are walked in a K order rotated by
 * tile column (the sum over K is then taken in another order than otherwise: still deterministic).  Whatever lies between a row's end and its leading dimension is never
 * used (NaN patterns there do not reach the result) and C's padding is never written; the library does
 * read, without using it, the rest of the 16-byte chunk that holds a row's last element.
 */
int gemm_select(int64_t M, int64_t N, int64_t K, int dtype, gemm_cfg *out);
/* The same for a given storage of B (gemm_select is b_layout = GEMM_B_ROW_MAJOR). */
int gemm_select_ex(int64_t M, int64_t N, int64_t K, int dtype, int b_layout, gemm_cfg *out);
/*
 * Strided-batched selection: `batch` independent products of one shape, C_b = alpha*A_b*B_b +
 * beta*C_b with X_b = X + b*stride_x (Sections II-B and V-C mention the batch dimension as a
 * multiplier of the tuning cost; here it multiplies the tile count of Algorithm 4).  The
 * whole batch is one launch (plus one reduction launch for split-K); Stream-K is not
 * offered for batch > 1.  1 <= batch <= 65535 (else GEMM_ERR_SHAPE).  gemm_run reads
 * batch and the strides from the cfg; strides must be multiples of 16 bytes (C: 8 elements).
 */
int gemm_select_batched(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int b_layout, gemm_cfg *out);
int gemm_cfg_at_batched(int idx, int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int b_layout,
                        gemm_cfg *out);

/*
 * Grouped GEMM: n_groups independent products C_g = alpha*A_g*B_g + beta*C_g of DIFFERENT shapes
 * (one dtype, one storage of B, one alpha and beta) in ONE launch of one kernel variant -- the
 * grouped dimension that Sections II-B and V-C name as a further multiplier of a tuning search
 * and that costs the analytical selector one more pass of the model over the groups.
 *
 *   gemm_problem      host-side description of one group.  M may be 0 (an empty group: nothing is
 *                     read or written, its pointers may be NULL); N, K >= 1.  A, B, C: device pointers,
 *                     16-byte aligned; ld* in elements, multiples of 16 bytes (ldc: of 8 elements).
 *                     gemm_select_grouped / gemm_cfg_at_grouped read M, N, K only.
 *   gemm_select_grouped  arg-min over the variants that are legal for every non-empty group (no
 *                     split-K, no Stream-K).  Model: Algorithm 4 counts the tiles of all groups
 *                     together, T = sum T_g, omega = ceil(T / workgroup slots); Algorithm 8 gives each
 *                     group its own tile latency L_tile(g) on a full device (its own cache tile,
 *                     hit rates and K loop); Algorithm 9 becomes omega * sum_g T_g L_tile(g) / T.
 *   gemm_cfg_at_grouped  the same for variant `variant` in [0, gemm_variant_count(dtype)), for sweeps.
 *   gemm_grouped_plan validates cfg and problems and writes n_groups table records (HOST memory,
 *                     caller-owned) and the launch's workgroup count.  With X = the descriptor's
 *                     XCD count (1 when cfg.xcd_remap = 0) a group of T tiles takes ceil(T / X)
 *                     consecutive slots on every XCD: workgroup p is slot p / X of XCD p % X, XCD x
 *                     computes the x-th of X contiguous chunks of the group's tiles, and a slot
 *                     beyond its chunk is idle.  Every group is thereby spread over all L2s.  The records are ordered by
 *                     descending K (ties: the caller's order), so that the longest tiles are
 *                     dispatched first; each carries its group's pointers.  The caller copies the
 *                     records, unchanged, to 16-byte aligned device memory.
 *   gemm_run_grouped  enqueues the launch.  host_table: the records gemm_grouped_plan wrote (checked
 *                     again); dev_table: their copy in device memory, which must stay unchanged
 *                     until the launch has finished.  Groups must not overlap in C.
 *   gemm_grouped_locate  host only: what workgroup `workgroup` of the launch computes, by the
 *                     kernel's own arithmetic: out3 = {record index, tile_m, tile_n}, or {-1,-1,-1}
 *                     for an idle slot.  GEMM_ERR_INDEX beyond the launch's workgroups.
 * 1 <= n_groups <= 4096.  Errors as for gemm_select / gemm_run; GEMM_ERR_CFG_ILLEGAL also when cfg
 * is not a grouped cfg for n_groups groups or a record does not belong to it.
 */
typedef struct gemm_problem {
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    const void *A;
    const void *B;
    void *C;
} gemm_problem;
typedef struct gemm_group_rec {
    uint64_t A, B, C;            /* device addresses */
    int32_t M, N, K;
    int32_t lda, ldb, ldc;
    int32_t tiles_m, tiles_n;    /* ceil(M / block_m), ceil(N / block_n) */
    int32_t tile_start;          /* first per-XCD slot of the group: sum of ceil(tiles / X) over the records before it */
    int32_t group_m;             /* band height of the group's rasterisation (Algorithm 6's f_m for its shape) */
} gemm_group_rec;                /* 64 bytes */
int gemm_select_grouped(int n_groups, const gemm_problem *problems, int dtype, int b_layout, gemm_cfg *out);
int gemm_cfg_at_grouped(int variant, int n_groups, const gemm_problem *problems, int dtype, int b_layout,
                        gemm_cfg *out);
int gemm_variant_count(int dtype);
int gemm_grouped_plan(const gemm_cfg *cfg, int n_groups, const gemm_problem *problems, gemm_group_rec *table_out,
                      int64_t *workgroups_out);
int gemm_grouped_locate(const gemm_cfg *cfg, int n_groups, const gemm_group_rec *table, int64_t workgroup,
                        int32_t out3[3]);
int gemm_run_grouped(const gemm_cfg *cfg, int n_groups, const gemm_group_rec *host_table, const void *dev_table,
                     void *hip_stream);

/*
 * Enqueue C = alpha * A * B + beta * C on hip_stream (a hipStream_t; NULL = the default stream) with
 * the kernel cfg names; returns without synchronising.  A, B, C: device pointers,
 * 16-byte aligned; lda, ldb multiples of 16 bytes, ldc a multiple of 8 elements (else GEMM_ERR_ALIGN).  When cfg->split_k > 1 or cfg->stream_k = 1 a workspace of
 * gemm_workspace_bytes(cfg) must have been registered with gemm_set_workspace for the
 * current device.
 */
int gemm_run(const gemm_cfg *cfg, const void *A, const void *B, void *C, void *hip_stream);

/*
 * gemm_run for callers that cannot allocate or register device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same launch, but split-K slabs and Stream-K
 * partial tiles go to a buffer of GEMM_NOALLOC_WORKSPACE_BYTES that is part of the library's code object
 * (one copy per GPU, held from module load until the process ends) instead of the registered workspace.
 * Calls no hipMalloc / hipFree and no allocating routine; the registered workspace is neither used nor
 * changed.  A cfg whose gemm_workspace_bytes exceeds GEMM_NOALLOC_WORKSPACE_BYTES returns
 * GEMM_ERR_WORKSPACE and launches nothing (cfgs with split_k = 1 and stream_k = 0 need no workspace and
 * always fit).  Every call on a GPU shares that GPU's buffer: the kernels overwrite what they later
 * read, so nothing has to be cleared between calls, but two calls in flight at once on one GPU (different
 * streams, or a captured graph replayed concurrently) race on it -- order them.  Other arguments and
 * errors as for gemm_run.
 */
#define GEMM_NOALLOC_WORKSPACE_BYTES (64u << 20)
int gemm_run_noalloc(const gemm_cfg *cfg, const void *A, const void *B, void *C, void *hip_stream);

/* fp32 partial sums: batch * split_k * M * ceil(N / 8) * 8 * 4 bytes when split_k > 1; 2 * sk_workers * block_m *
 * block_n * 4 bytes (two partial tiles per stream-K workgroup) when stream_k = 1; else 0. */
size_t gemm_workspace_bytes(const gemm_cfg *cfg);

/*
 * Stream-K work split of a cfg with stream_k = 1 (Section V-E: the paper's kernels use
 * Stream-K against wave quantisation).  Host only, no GPU: the same arithmetic the kernel
 * runs, exposed for tests and tools.  Tiles are taken in rasterisation order; the first
 * dp_tiles get one workgroup each, the last sk_tiles = tiles % sk_workers are cut along K:
 * with S = ceil(K / block_k) slabs per tile, worker g owns iterations
 * [g * sk_tiles * S / G, (g + 1) * sk_tiles * S / G) of the tile-major numbering.
 *   gemm_stream_k_plan      writes {workers G, sk_tiles, dp_tiles, slabs S} to plan4.
 *   gemm_stream_k_segments  writes worker g's segments (at most 2) and returns their number
 *                           (>= 0) or a negative gemm_status.  A segment with complete = 1 is
 *                           stored to C by its worker; any other leaves an fp32 partial tile in
 *                           workspace slot 2 * g + (segment number) for the summation pass.
 *   gemm_stream_k_contributors  what the summation pass adds up for stream-K tile j: writes
 *                           {first worker, last worker, segment number of the first worker's
 *                           partial} to out3; the partials of the later workers are their
 *                           segment 0.  first == last means one worker stored the whole tile.
 * Errors: GEMM_ERR_NULL, GEMM_ERR_ABI, GEMM_ERR_CFG_ILLEGAL (not a legal stream-K cfg),
 * GEMM_ERR_INDEX (worker outside [0, G), tile outside [0, sk_tiles)).
 */
typedef struct gemm_sk_segment {
    int32_t tile_m, tile_n;   /* output tile coordinates */
    int32_t slab0, count;     /* K_T slabs [slab0, slab0 + count) of the tile */
    int32_t complete;         /* 1: the whole tile */
    int32_t sk_tile;          /* index among the stream-K tiles */
} gemm_sk_segment;
int gemm_stream_k_plan(const gemm_cfg *cfg, int32_t plan4[4]);
int gemm_stream_k_segments(const gemm_cfg *cfg, int worker, gemm_sk_segment seg[2]);
int gemm_stream_k_contributors(const gemm_cfg *cfg, int sk_tile, int32_t out3[3]);

/* Register (or, with NULL/0, drop) a caller-owned device buffer used by split-K and stream-K runs.
 * The buffer must outlive every gemm_run that uses it; runs that share it must be
 * stream-ordered. */
int gemm_set_workspace(void *dev_ptr, size_t bytes);

/* Enumeration of the compiled configuration space, for the offline sweep only:
 * idx in [0, gemm_cfg_count(dtype)).  gemm_cfg_at returns GEMM_ERR_CFG_ILLEGAL when
 * variant idx cannot run the shape (e.g. more K slices than K slabs). */
int gemm_cfg_count(int dtype);
int gemm_cfg_at(int idx, int64_t M, int64_t N, int64_t K, int dtype, gemm_cfg *out);
int gemm_cfg_at_ex(int idx, int64_t M, int64_t N, int64_t K, int dtype, int b_layout, gemm_cfg *out);

/* Model terms for a cfg (Algorithms 3-9), host only. */
int gemm_predict(const gemm_cfg *cfg, gemm_prediction *out);

/*
 * Diagnostic (needs the GPU, not part of selection): the number of workgroups of compiled variant
 * `variant` in [0, gemm_variant_count(dtype)) that the HIP runtime reports as resident on one CU
 * (registers, LDS and wave slots of the actual code object) -- what gemm_prediction.occupancy
 * estimates on the host.  Errors: GEMM_ERR_NULL, GEMM_ERR_DTYPE, GEMM_ERR_INDEX,
 * GEMM_ERR_CFG_ILLEGAL (b_layout), GEMM_ERR_HIP.
 */
int gemm_variant_occupancy(int dtype, int variant, int b_layout, int *blocks_per_cu);

/* Hardware descriptor: get a copy / replace it (process-wide; not thread-safe against
 * concurrent gemm_select).  gemm_hw_reset restores the MI355X defaults. */
int gemm_hw_get(gemm_hw *out);
int gemm_hw_set(const gemm_hw *in);
int gemm_hw_reset(void);

/*
 * Built-in descriptors (Section I: porting the selector to another GPU is a matter of
 * replacing the hardware table; Section V evaluates on a 304-CU part).  Writes the table to
 * *out without installing it; pass it to gemm_hw_set to retarget gemm_select / gemm_predict.
 *   GEMM_HW_MI355X       the default: 256 CUs in 8 XCDs, 160 KB LDS, measured rates.
 *   GEMM_HW_MI300X_LIKE  304 CUs in 8 XCDs of 38, 64 KB LDS, 4 MB L2 per XCD, 256 MB MALL,
 *                        2.1 GHz, public bandwidth figures, matrix-instruction intervals of
 *                        the half-rate CDNA3 matrix cores.  For the selector only: the kernels
 *                        of this library are gfx950 code, and variants whose LDS ring exceeds
 *                        64 KB are not candidates under this table.
 * Errors: GEMM_ERR_NULL, GEMM_ERR_INDEX (unknown id).
 */
typedef enum { GEMM_HW_MI355X = 0, GEMM_HW_MI300X_LIKE = 1 } gemm_hw_id;
int gemm_hw_preset(int id, gemm_hw *out);

/*
 * Calibration probes (Section I: the model's hardware rates come from micro-benchmarks).
 * Each launches its kernel on hip_stream at least twice, times the later launches with HIP events,
 * synchronises and writes the measured rate.  scratch4: caller-owned device memory, at least 4 bytes.
 *   gemm_probe_mfma   register-resident MFMA loop on constant operands for (dtype, mfma in {32, 16}),
 *                     10 ms untimed then 10 ms timed (gemm_probe_mfma_ex with operands = 0) -> TFLOP/s
 *                     on the whole device; L_MI in clocks = flop per instruction * n_cu * simd_per_cu *
 *                     clk_ghz / (TFLOP/s * 1e3).
 *   gemm_probe_stream streaming 128-bit reads of buf[0, bytes) (device memory, 16-byte aligned,
 *                     >= 1 MiB; use more than the 256 MiB MALL to measure HBM) -> GB/s.
 */
int gemm_probe_mfma(int dtype, int mfma, void *scratch4, void *hip_stream, double *tflops_out);
int gemm_probe_stream(const void *buf, size_t bytes, void *scratch4, void *hip_stream, double *gbps_out);
/*
 * Further probes, one per remaining measurable entry of the hardware descriptor (Section I; Section IV's
 * H: the rates R_1, R_2, R_MEM and the latency L_lat of Algorithm 7, L_MI of Algorithm 3).  Same
 * conventions: synchronous, self-timed, scratch4 = caller-owned device memory of at least 4 bytes.
 *   gemm_probe_mfma_ex   the matrix-core ceiling on a workload's own operand statistics.  A wave keeps
 *                        2 register sets of 2-4 column and 4 row fragments and accumulates their
 *                        products in turn, as the GEMM kernel's k-steps do.  operands = 0: every
 *                        element 1.0; operands = 1: per-lane different N(0,1) values (bf16), or N(0,1)
 *                        scaled to a maximum of 448 (e4m3), so the datapath toggles as on the benchmark
 *                        inputs.  Launches run untimed for about warm_ms, then timed for about
 *                        timed_ms (each in (0, 1000]; warm_ms may be 0): the chip needs 15-20 ms of
 *                        work after an idle gap to settle under its power limit.  -> TFLOP/s.
 *   gemm_probe_read      `passes` (1 .. 4096) reads of buf[0, bytes) by one launch, every workgroup
 *                        re-reading its own grid-strided share.  Which level serves the repeats follows
 *                        from the size: up to about 2 MiB per L2 (16 MiB on 8 XCDs) the L2s, up to the
 *                        MALL's capacity the MALL, beyond it HBM.  -> GB/s over all passes.
 *   gemm_probe_lds       LDS fragment-read rate with `waves_per_cu` in {4, 8, 16} waves per CU reading
 *                        conflict-free: kind 0 ds_read_b128, 1 ds_read_b64, 2 ds_read_b64_tr_b16,
 *                        3 ds_read_b64_tr_b8.  -> GB/s over the whole device (divide by CUs and clock
 *                        for bytes per clock and CU).
 *   gemm_probe_fill      the GEMM kernel's refill in isolation: one or two (`wgs_per_cu`) workgroups of 8
 *                        waves per CU move 64 KiB slabs from buf towards LDS, 16 bytes per lane and
 *                        request, two slabs in flight, with a workgroup barrier per slab when `sync` is
 *                        non-zero.  kind 0: buffer loads that write LDS directly; 1: the same 4 bytes per
 *                        lane; 2: loads into registers only; 3: loads into registers, then ds_write_b128.
 *                        pattern 0: slabs of consecutive bytes inside the first `footprint` bytes of buf
 *                        (a power of two, 64 KiB .. 2 GiB, <= bytes; its size decides the level that
 *                        serves them); pattern 1: slabs of 512 rows of 128 bytes, 16 KiB apart (a K slab
 *                        of a row-major bf16 operand with K = 8192), stepping along the first `footprint`
 *                        bytes (128 .. 16384, a power of two) of the rows; bytes >= 8 MiB.  patterns 2
 *                        and 3 (not with kind 1): slabs of 512 pieces of 128 bytes / 128 pieces of 512
 *                        bytes of consecutive rows 16 KiB apart, walking the first `footprint` bytes of
 *                        buf (a power of two, 8 MiB .. 2 GiB, <= bytes) so that every byte is read once
 *                        before any is read again: the operand traffic of a large GEMM beyond the L2.
 *                        buf is 128-byte aligned device memory, only read.  -> GB/s over the whole device.
 *   gemm_probe_latency   4096 dependent loads by one lane through buf[0, bytes) (device memory,
 *                        128-byte aligned, >= 1 MiB; OVERWRITTEN with the chain), every hop on another
 *                        128-byte line; the level that holds the chain follows from the size as for
 *                        gemm_probe_read.  -> nanoseconds per load.
 * Errors: GEMM_ERR_NULL, GEMM_ERR_DTYPE, GEMM_ERR_CFG_ILLEGAL (mfma, operands, kind, waves, times),
 * GEMM_ERR_ALIGN (buffer too small or misaligned), GEMM_ERR_SHAPE (passes), GEMM_ERR_HIP.
 */
int gemm_probe_mfma_ex(int dtype, int mfma, int operands, double warm_ms, double timed_ms, void *scratch4,
                       void *hip_stream, double *tflops_out);
int gemm_probe_read(const void *buf, size_t bytes, int passes, void *scratch4, void *hip_stream, double *gbps_out);
int gemm_probe_lds(int kind, int waves_per_cu, void *scratch4, void *hip_stream, double *gbps_out);
int gemm_probe_fill(int kind, int pattern, int wgs_per_cu, int sync, const void *buf, size_t bytes, size_t footprint,
                    void *scratch4, void *hip_stream, double *gbps_out);
int gemm_probe_latency(void *buf, size_t bytes, void *scratch4, void *hip_stream, double *ns_out);

#ifdef __cplusplus
}
#endif
#endif /* GEMM355_GEMM_H */
