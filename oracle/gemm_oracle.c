/*
 * CPU oracle for C = alpha * A * B  (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the reference the GPU kernels are checked against.  It is plain,
 * slow C and shares no code with the HIP path.  Only tests, the smoke check and
 * the bench's cpu_baseline leg may call it; the product never does.
 *
 * What it computes: the paper's Section II-A definition C = alpha*A*B + beta*C
 * with beta = 0, evaluated exactly as the paper's Algorithm 1 states it -- for
 * every output element, a running sum over the reduction index in ascending
 * order -- in fp64.  Inputs are bf16, IEEE binary16 ("fp16": 1-5-10, bias 15;
 * the precision of the paper's own runs, Section V) or OCP fp8 e4m3 ("e4m3fn":
 * 1-4-3, bias 7, no infinities, S.1111.111 is NaN, largest finite 448) bit
 * patterns decoded exactly; a product of two such values is exact in fp64, so
 * the only rounding is the fp64 accumulation (relative error <= K * 2^-53) and
 * the final round-to-nearest-even to the output format: bf16, or fp16 when the
 * inputs are fp16.
 *
 * Pins (tests/test_oracle_*.py): identity, permutations, rank-1 closed forms,
 * exact small-integer sums against an integer-only computation, codec
 * round-trips over every bf16 / e4m3 code, and the literal Algorithm-1 loop
 * nest against the row-accumulating loop nest.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_BF16 0
#define ORACLE_E4M3 1
#define ORACLE_FP16 2

/* ---- decoders: bit pattern -> exact fp64 value (from the format definitions) ---- */

double oracle_bf16_to_f64(uint16_t bits)
{
    int sign = bits >> 15;
    int e = (bits >> 7) & 0xFF;
    int m = bits & 0x7F;
    double v;
    if (e == 0xFF)
        v = m ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)m, -126 - 7);          /* subnormal: m * 2^-133 */
    else
        v = ldexp((double)(128 + m), e - 127 - 7); /* (1 + m/128) * 2^(e-127) */
    return sign ? -v : v;
}

/* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double oracle_fp16_to_f64(uint16_t bits)
{
    int sign = bits >> 15;
    int e = (bits >> 10) & 0x1F;
    int m = bits & 0x3FF;
    double v;
    if (e == 0x1F)
        v = m ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)m, -14 - 10);            /* subnormal: m * 2^-24 */
    else
        v = ldexp((double)(1024 + m), e - 15 - 10); /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

double oracle_e4m3_to_f64(uint8_t bits)
{
    int sign = bits >> 7;
    int e = (bits >> 3) & 0xF;
    int m = bits & 0x7;
    double v;
    if (e == 0xF && m == 0x7)
        v = NAN;                                  /* the only non-finite code */
    else if (e == 0)
        v = ldexp((double)m, -6 - 3);             /* subnormal: m * 2^-9 */
    else
        v = ldexp((double)(8 + m), e - 7 - 3);    /* (1 + m/8) * 2^(e-7) */
    return sign ? -v : v;
}

/* ---- encoders: fp64 -> nearest code, ties to even ---- */

/* Round |x| to a grid with `mant` explicit mantissa bits and smallest normal
 * exponent `emin`; returns the rounded magnitude (exact in fp64). */
static double round_to_format(double ax, int mant, int emin)
{
    int ex;
    if (ax == 0.0)
        return 0.0;
    frexp(ax, &ex);               /* ax = f * 2^ex, f in [0.5,1)  => floor(log2 ax) = ex-1 */
    int e = ex - 1;
    if (e < emin)
        e = emin;                 /* subnormal range shares the ulp of the smallest normal */
    int q = e - mant;             /* exponent of one unit in the last place */
    double scaled = ldexp(ax, -q);   /* exact */
    double r = nearbyint(scaled);    /* default rounding mode: nearest, ties to even */
    return ldexp(r, q);
}

uint16_t oracle_f64_to_bf16(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0;
    if (isnan(x))
        return 0x7FC0u;
    double ax = fabs(x);
    if (isinf(ax))
        return sign | 0x7F80u;
    double r = round_to_format(ax, 7, -126);
    if (r >= ldexp(1.0, 128))
        return sign | 0x7F80u;    /* rounds past the largest finite bf16 */
    /* r is representable in bf16, hence in fp32: its fp32 pattern has zero low half */
    float f = (float)r;
    uint32_t u;
    memcpy(&u, &f, 4);
    return sign | (uint16_t)(u >> 16);
}

/* fp64 -> binary16, round-to-nearest-even; what rounds to 2^16 or beyond becomes infinity. */
uint16_t oracle_f64_to_fp16(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0;
    if (isnan(x))
        return 0x7E00u;
    double ax = fabs(x);
    if (isinf(ax))
        return sign | 0x7C00u;
    double r = round_to_format(ax, 10, -14);
    if (r >= 65536.0)
        return sign | 0x7C00u;
    if (r == 0.0)
        return sign;
    int ex;
    double f = frexp(r, &ex);     /* r = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;
    if (e < -14)                  /* subnormal: r = m * 2^-24 */
        return sign | (uint16_t)ldexp(r, 24);
    int m = (int)ldexp(f, 11) - 1024;   /* 2f in [1,2): 2f = 1 + m/1024 */
    return sign | (uint16_t)(((e + 15) << 10) | m);
}

/* fp64 -> e4m3fn, round-to-nearest-even, magnitudes beyond 448 saturate to 448. */
uint8_t oracle_f64_to_e4m3(double x)
{
    uint8_t sign = signbit(x) ? 0x80u : 0;
    if (isnan(x))
        return sign | 0x7Fu;
    double ax = fabs(x);
    double r = isinf(ax) ? 448.0 : round_to_format(ax, 3, -6);
    if (r > 448.0)
        r = 448.0;
    if (r == 0.0)
        return sign;
    int ex;
    double f = frexp(r, &ex);     /* r = f * 2^ex */
    int e = ex - 1;
    if (e < -6) {                 /* subnormal: r = m * 2^-9 */
        int m = (int)ldexp(r, 9);
        return sign | (uint8_t)m;
    }
    int m = (int)ldexp(f, 4) - 8; /* f*2 in [1,2): (1+m/8) => f*16 = 8+m */
    return sign | (uint8_t)(((e + 7) << 3) | m);
}

/* Value tables filled once from the two decoders above (every code of each format). */
static double bf16_table[65536];
static double fp16_table[65536];
static double e4m3_table[256];
static int tables_ready = 0;

static void fill_tables(void)
{
    if (tables_ready)
        return;
    for (int c = 0; c < 65536; ++c)
        bf16_table[c] = oracle_bf16_to_f64((uint16_t)c);
    for (int c = 0; c < 65536; ++c)
        fp16_table[c] = oracle_fp16_to_f64((uint16_t)c);
    for (int c = 0; c < 256; ++c)
        e4m3_table[c] = oracle_e4m3_to_f64((uint8_t)c);
    tables_ready = 1;
}

static inline double decode(const void *p, int64_t idx, int dtype)
{
    if (dtype == ORACLE_BF16)
        return bf16_table[((const uint16_t *)p)[idx]];
    if (dtype == ORACLE_FP16)
        return fp16_table[((const uint16_t *)p)[idx]];
    return e4m3_table[((const uint8_t *)p)[idx]];
}

static inline int known_dtype(int dtype) { return dtype == ORACLE_BF16 || dtype == ORACLE_E4M3 || dtype == ORACLE_FP16; }

/* The 16-bit output code: fp16 for fp16 inputs, bf16 otherwise. */
static inline uint16_t encode_out(double c, int dtype)
{
    return dtype == ORACLE_FP16 ? oracle_f64_to_fp16(c) : oracle_f64_to_bf16(c);
}

/*
 * Algorithm 1 verbatim in structure: i, then j, then the reduction index
 * ascending.  A is M x K row-major (leading dimension lda), B is K x N
 * row-major (ldb).  Writes alpha * sum as fp64 (C64, ld = N, may be NULL) and
 * its rounding to the 16-bit output format (C16, ld = ldc, may be NULL).  Returns 0, or -1 on bad
 * arguments.
 */
int oracle_gemm_alg1(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                     int64_t ldb, int dtype, double alpha, uint16_t *C16, int64_t ldc, double *C64)
{
    if (M < 0 || N < 0 || K < 0 || !known_dtype(dtype))
        return -1;
    fill_tables();
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double c = 0.0;
            for (int64_t l = 0; l < K; ++l)
                c = c + decode(A, i * lda + l, dtype) * decode(B, l * ldb + j, dtype);
            c = alpha * c;
            if (C64)
                C64[i * N + j] = c;
            if (C16)
                C16[i * ldc + j] = encode_out(c, dtype);
        }
    return 0;
}

/*
 * Same sums, loop nest i / reduction index / j so that B is walked along its
 * rows: every C[i,j] still receives its K products in ascending order of the
 * reduction index, so each result equals oracle_gemm_alg1's bit for bit.  Rows
 * are independent and are spread over OpenMP threads.
 */
int oracle_gemm(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                int64_t ldb, int dtype, double alpha, uint16_t *C16, int64_t ldc, double *C64)
{
    if (M < 0 || N < 0 || K < 0 || !known_dtype(dtype))
        return -1;
    fill_tables();
    int failed = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double *brow = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        if (!acc || !brow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < M; ++i) {
            if (failed)
                continue;
            for (int64_t j = 0; j < N; ++j)
                acc[j] = 0.0;
            for (int64_t l = 0; l < K; ++l) {
                double a = decode(A, i * lda + l, dtype);
                for (int64_t j = 0; j < N; ++j)
                    brow[j] = decode(B, l * ldb + j, dtype);
                for (int64_t j = 0; j < N; ++j)
                    acc[j] = acc[j] + a * brow[j];
            }
            for (int64_t j = 0; j < N; ++j) {
                double c = alpha * acc[j];
                if (C64)
                    C64[i * N + j] = c;
                if (C16)
                    C16[i * ldc + j] = encode_out(c, dtype);
            }
        }
        free(acc);
        free(brow);
    }
    return failed ? -2 : 0;
}

/*
 * Selected rows only (for full-size checks where the whole product would take
 * too long): out row r holds row rows[r] of the product.  C16/C64 are
 * n_rows x N, densely packed.
 */
int oracle_gemm_rows(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                     int64_t ldb, int dtype, double alpha, int64_t n_rows, const int64_t *rows,
                     uint16_t *C16, double *C64)
{
    if (M < 0 || N < 0 || K < 0 || n_rows < 0 || !known_dtype(dtype))
        return -1;
    for (int64_t r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= M)
            return -1;
    fill_tables();
    int failed = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        if (!acc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            if (failed)
                continue;
            int64_t i = rows[r];
            for (int64_t j = 0; j < N; ++j)
                acc[j] = 0.0;
            for (int64_t l = 0; l < K; ++l) {
                double a = decode(A, i * lda + l, dtype);
                for (int64_t j = 0; j < N; ++j)
                    acc[j] = acc[j] + a * decode(B, l * ldb + j, dtype);
            }
            for (int64_t j = 0; j < N; ++j) {
                double c = alpha * acc[j];
                if (C64)
                    C64[r * N + j] = c;
                if (C16)
                    C16[r * N + j] = encode_out(c, dtype);
            }
        }
        free(acc);
    }
    return failed ? -2 : 0;
}

/* Selected elements (rows[s], cols[s]), each by its own Algorithm-1 inner loop. */
int oracle_gemm_samples(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                        int64_t ldb, int dtype, double alpha, int64_t n, const int64_t *rows,
                        const int64_t *cols, uint16_t *C16, double *C64)
{
    if (M < 0 || N < 0 || K < 0 || n < 0 || !known_dtype(dtype))
        return -1;
    for (int64_t s = 0; s < n; ++s)
        if (rows[s] < 0 || rows[s] >= M || cols[s] < 0 || cols[s] >= N)
            return -1;
    fill_tables();
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t s = 0; s < n; ++s) {
        double c = 0.0;
        for (int64_t l = 0; l < K; ++l)
            c = c + decode(A, rows[s] * lda + l, dtype) * decode(B, l * ldb + cols[s], dtype);
        c = alpha * c;
        if (C64)
            C64[s] = c;
        if (C16)
            C16[s] = encode_out(c, dtype);
    }
    return 0;
}

/* Bulk codecs for the tests. */
void oracle_decode_bf16(int64_t n, const uint16_t *in, double *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = oracle_bf16_to_f64(in[i]);
}
void oracle_decode_fp16(int64_t n, const uint16_t *in, double *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = oracle_fp16_to_f64(in[i]);
}
void oracle_encode_fp16(int64_t n, const double *in, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = oracle_f64_to_fp16(in[i]);
}
void oracle_decode_e4m3(int64_t n, const uint8_t *in, double *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = oracle_e4m3_to_f64(in[i]);
}
void oracle_encode_bf16(int64_t n, const double *in, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = oracle_f64_to_bf16(in[i]);
}
void oracle_encode_e4m3(int64_t n, const double *in, uint8_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = oracle_f64_to_e4m3(in[i]);
}
