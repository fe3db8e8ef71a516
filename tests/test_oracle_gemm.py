"""Pins for the CPU GEMM oracle: facts fixed by the format definitions and by
linear algebra, none of them computed by the oracle's own formulae."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

BF16, E4M3 = 0, 1


# ---------- codecs ----------

def test_bf16_decode_every_code_matches_fp32_view(oracle):
    codes = np.arange(65536, dtype=np.uint16)
    got = oracle.decode_bf16(codes)
    ref = (codes.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_bf16_encode_roundtrip_every_finite_code(oracle):
    codes = np.arange(65536, dtype=np.uint16)
    vals = oracle.decode_bf16(codes)
    fin = np.isfinite(vals)
    assert np.array_equal(oracle.encode_bf16(vals[fin]), codes[fin])


def test_bf16_encode_ties_to_even_and_integers(oracle):
    # bf16 keeps 8 significant bits: integers above 256 round to multiples of 2, 4, ...
    x = np.array([255, 256, 257, 258, 259, 260, 261, 513, 514, 515, 518, -257, -259, 8191, 8192],
                 dtype=np.float64)
    want = np.array([255, 256, 256, 258, 260, 260, 260, 512, 512, 516, 520, -256, -260, 8192, 8192],
                    dtype=np.float64)
    got = oracle.decode_bf16(oracle.encode_bf16(x))
    assert np.array_equal(got, want)
    # exact ties around 1.0 (ulp 2^-7): 1+2^-8 -> 1 (even), 1+3*2^-8 -> 1+2^-6 (even mantissa 2)
    t = np.array([1 + 2.0**-8, 1 + 3 * 2.0**-8, 1 + 2.0**-8 + 2.0**-30, 1 + 2.0**-8 - 2.0**-30])
    w = np.array([1.0, 1 + 2.0**-6, 1 + 2.0**-7, 1.0])
    assert np.array_equal(oracle.decode_bf16(oracle.encode_bf16(t)), w)


def test_bf16_encode_random_matches_single_rounding_via_integers(oracle):
    # independent route: for |x| in [2^e, 2^e+1) the bf16 grid is 2^(e-7); use python ints/fractions
    from fractions import Fraction
    g = np.random.default_rng(11)
    xs = g.standard_normal(2000) * np.exp(g.uniform(-20, 20, 2000))
    got = oracle.decode_bf16(oracle.encode_bf16(xs))
    for x, y in zip(xs, got):
        fx = Fraction(float(abs(x)))
        e = int(np.floor(np.log2(abs(x))))
        while Fraction(2) ** e > fx:
            e -= 1
        while Fraction(2) ** (e + 1) <= fx:
            e += 1
        ulp = Fraction(2) ** (e - 7)
        q = fx / ulp
        lo = q.numerator // q.denominator
        rem = q - lo
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
            lo += 1
        assert Fraction(float(abs(y))) == lo * ulp
        assert np.sign(x) == np.sign(y)


def test_e4m3_decode_every_code_matches_torch(oracle):
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.decode_e4m3(codes)
    ref = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    nan = np.isnan(ref)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    # format facts: largest finite 448, smallest subnormal 2^-9, smallest normal 2^-6
    assert got[0x7E] == 448.0 and got[0x01] == 2.0**-9 and got[0x08] == 2.0**-6


def test_e4m3_encode_roundtrip_and_torch_cast(oracle):
    codes = np.arange(256, dtype=np.uint8)
    vals = oracle.decode_e4m3(codes)
    fin = np.isfinite(vals)
    assert np.array_equal(oracle.encode_e4m3(vals[fin]), codes[fin])
    g = np.random.default_rng(5)
    x = (g.standard_normal(20000) * np.exp(g.uniform(-8, 5, 20000))).astype(np.float32)
    x = np.clip(x, -448, 448)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.encode_e4m3(x.astype(np.float64))
    assert np.array_equal(got, ref)
    # ties: 17 lies midway between 16 and 18 -> 16 (even mantissa); 19 -> 20; beyond 448 saturates
    t = oracle.decode_e4m3(oracle.encode_e4m3(np.array([17.0, 19.0, 1000.0, -1e9, 2.0**-10, 3 * 2.0**-10])))
    assert np.array_equal(t, np.array([16.0, 20.0, 448.0, -448.0, 0.0, 2.0**-8]))


def test_workload_quantizer_agrees_with_oracle_encoder(oracle):
    g = np.random.default_rng(9)
    x = g.standard_normal((64, 48)).astype(np.float32)
    codes, s = wl.quantize_e4m3(x)
    assert np.array_equal(codes, oracle.encode_e4m3((x / s).astype(np.float64)))
    assert np.max(np.abs(oracle.decode_e4m3(codes))) == 448.0


# ---------- GEMM: closed forms ----------

def _bf16(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _eye_bits(n, dtype):
    one = 0x3F80 if dtype == BF16 else 0x38
    t = np.uint16 if dtype == BF16 else np.uint8
    return (np.eye(n, dtype=np.int64) * one).astype(t)


@pytest.mark.parametrize("dtype", [BF16, E4M3])
def test_identity(oracle, dtype):
    g = np.random.default_rng(1)
    M, K = 37, 53
    if dtype == BF16:
        A = _bf16(g.standard_normal((M, K)))
        want = A
    else:
        A = g.integers(0, 256, size=(M, K)).astype(np.uint8)
        A[(A & 0x7F) == 0x7F] = 0x10          # no NaN codes
        want = oracle.encode_bf16(oracle.decode_e4m3(A))   # every e4m3 value is a bf16 value
    C16, C64 = oracle.gemm(A, _eye_bits(K, dtype), dtype)
    assert np.array_equal(C64, oracle.decode(A, dtype))
    got, ref = C16.copy(), want.copy()
    got[got == 0x8000] = 0                      # -0 * 1 + 0 = +0 in a running sum
    ref[ref == 0x8000] = 0
    assert np.array_equal(got, ref)
    B = A.T.copy()
    C16b, C64b = oracle.gemm(_eye_bits(K, dtype), B, dtype)
    assert np.array_equal(C64b, oracle.decode(B, dtype))


def test_permutation_right_and_left(oracle):
    g = np.random.default_rng(2)
    M, K, N = 19, 23, 23
    A = _bf16(g.standard_normal((M, K)))
    perm = g.permutation(K)
    P = np.zeros((K, N), np.uint16)
    P[perm, np.arange(N)] = 0x3F80              # column j of A.P is column perm[j] of A
    C16, C64 = oracle.gemm(A, P, BF16)
    assert np.array_equal(C64, oracle.decode_bf16(A)[:, perm])
    B = _bf16(g.standard_normal((K, 31)))
    Q = np.zeros((K, K), np.uint16)
    Q[np.arange(K), perm] = 0x3F80              # row i of Q.B is row perm[i] of B
    C16, C64 = oracle.gemm(Q, B, BF16)
    assert np.array_equal(C64, oracle.decode_bf16(B)[perm, :])


def test_rank1_outer_product_k1(oracle):
    # K = 1: C[i,j] = a_i * b_j; powers of two times small odd integers stay exact in bf16
    a = np.array([1, -2, 3, 0.5, -0.25, 6, 12, 0], dtype=np.float32)
    b = np.array([1, 5, -7, 0.125, 10, -3], dtype=np.float32)
    A = _bf16(a.reshape(-1, 1))
    B = _bf16(b.reshape(1, -1))
    C16, C64 = oracle.gemm(A, B, BF16)
    want = np.outer(a.astype(np.float64), b.astype(np.float64))
    assert np.array_equal(C64, want)
    assert np.array_equal(wl.bf16_bits_to_f32(C16).astype(np.float64), want)   # all products fit 8 bits


def test_rank1_constant_along_k(oracle):
    # A[i,l] = u_i, B[l,j] = v_j  =>  C[i,j] = K u_i v_j   (asymmetric shapes catch a transpose)
    K = 96
    u = np.array([1, 2, -4, 0.5, 8], dtype=np.float32)
    v = np.array([1, -1, 2, 0.25, 4, -8, 16], dtype=np.float32)
    A = _bf16(np.repeat(u[:, None], K, axis=1))
    B = _bf16(np.repeat(v[None, :], K, axis=0))
    C16, C64 = oracle.gemm(A, B, BF16)
    want = K * np.outer(u.astype(np.float64), v.astype(np.float64))
    assert C64.shape == (5, 7) and np.array_equal(C64, want)
    assert np.array_equal(wl.bf16_bits_to_f32(C16).astype(np.float64), want)   # 96 = 3 * 32 fits


def _int_to_bf16_value(v):
    """Nearest-even rounding of a python int to 8 significant bits, by integer arithmetic only."""
    s, a = (-1 if v < 0 else 1), abs(v)
    if a < 256:
        return float(v)
    shift = a.bit_length() - 8
    q, r = a >> shift, a & ((1 << shift) - 1)
    half = 1 << (shift - 1)
    if r > half or (r == half and (q & 1)):
        q += 1
    return float(s * (q << shift))


@pytest.mark.parametrize("shape", [(8, 8, 8), (5, 7, 3), (33, 17, 129), (64, 48, 512)])
def test_small_integers_exact(oracle, shape):
    M, N, K = shape
    A, B = wl.integer_bf16(M, N, K, seed=7, case=K)
    Ai = wl.bf16_bits_to_f32(A).astype(np.int64)
    Bi = wl.bf16_bits_to_f32(B).astype(np.int64)
    want = np.zeros((M, N), dtype=np.int64)
    for i in range(M):                          # brute force in integers
        for j in range(N):
            want[i, j] = int(np.sum(Ai[i, :] * Bi[:, j]))
    C16, C64 = oracle.gemm(A, B, BF16)
    assert np.array_equal(C64, want.astype(np.float64))
    want16 = np.vectorize(_int_to_bf16_value)(want)
    assert np.array_equal(wl.bf16_bits_to_f32(C16).astype(np.float64), want16)
    if K == 512:
        assert np.abs(want).max() > 256          # the rounding branch is exercised


def test_literal_alg1_equals_row_walk_bitwise(oracle):
    A, B = wl.uniform_bf16(29, 41, 67, seed=3)
    a16, a64 = oracle.gemm(A, B, BF16, alpha=0.375, literal=True)
    b16, b64 = oracle.gemm(A, B, BF16, alpha=0.375)
    assert np.array_equal(a64.view(np.uint64), b64.view(np.uint64)) and np.array_equal(a16, b16)
    Aq, Bq, sa, sb = wl.normal_e4m3(13, 21, 40, seed=3)
    a16, a64 = oracle.gemm(Aq, Bq, E4M3, alpha=float(sa) * float(sb), literal=True)
    b16, b64 = oracle.gemm(Aq, Bq, E4M3, alpha=float(sa) * float(sb))
    assert np.array_equal(a64.view(np.uint64), b64.view(np.uint64)) and np.array_equal(a16, b16)


@pytest.mark.parametrize("dtype", [BF16, E4M3])
def test_random_matches_numpy_fp64_matmul(oracle, dtype):
    M, N, K = 45, 38, 301
    if dtype == BF16:
        A, B = wl.uniform_bf16(M, N, K, seed=21)
        alpha = 1.0
    else:
        A, B, sa, sb = wl.normal_e4m3(M, N, K, seed=21)
        alpha = float(sa) * float(sb)
    C16, C64 = oracle.gemm(A, B, dtype, alpha=alpha)
    ref = alpha * (oracle.decode(A, dtype) @ oracle.decode(B, dtype))
    scale = np.abs(ref).max()
    assert np.max(np.abs(C64 - ref)) <= 1e-12 * scale
    # bf16 output within half an ulp (2^-8 relative) of the fp64 value
    out = wl.bf16_bits_to_f32(C16).astype(np.float64)
    assert np.all(np.abs(out - C64) <= 2.0**-8 * np.abs(C64) + 1e-300)


def test_alpha_and_linearity(oracle):
    A, B = wl.uniform_bf16(16, 24, 64, seed=5)
    _, c1 = oracle.gemm(A, B, BF16, alpha=1.0)
    _, c4 = oracle.gemm(A, B, BF16, alpha=4.0)
    _, cm = oracle.gemm(A, B, BF16, alpha=-0.5)
    assert np.array_equal(c4, 4.0 * c1) and np.array_equal(cm, -0.5 * c1)
    # splitting K: A.B = A[:, :k].B[:k] + A[:, k:].B[k:]  (fp64, to rounding)
    _, lo = oracle.gemm(A[:, :40].copy(), B[:40].copy(), BF16)
    _, hi = oracle.gemm(A[:, 40:].copy(), B[40:].copy(), BF16)
    assert np.max(np.abs(lo + hi - c1)) <= 1e-13 * np.abs(c1).max() * 64


def test_rows_and_samples_agree_with_full(oracle):
    A, B = wl.uniform_bf16(40, 33, 77, seed=6)
    C16, C64 = oracle.gemm(A, B, BF16, alpha=2.0)
    rows = np.array([0, 39, 7, 7])
    r16, r64 = oracle.gemm_rows(A, B, rows, BF16, alpha=2.0)
    assert np.array_equal(r16, C16[rows]) and np.array_equal(r64, C64[rows])
    g = np.random.default_rng(0)
    rr, cc = g.integers(0, 40, 50), g.integers(0, 33, 50)
    s16, s64 = oracle.gemm_samples(A, B, rr, cc, BF16, alpha=2.0)
    assert np.array_equal(s16, C16[rr, cc]) and np.array_equal(s64, C64[rr, cc])


def test_empty_and_bad_arguments(oracle):
    A = np.zeros((3, 0), np.uint16)
    B = np.zeros((0, 4), np.uint16)
    C16, C64 = oracle.gemm(A, B, BF16)
    assert C16.shape == (3, 4) and not C16.any() and not C64.any()
    with pytest.raises(ValueError):
        oracle.gemm(np.zeros((3, 2), np.uint16), np.zeros((3, 2), np.uint16), BF16)
    with pytest.raises(TypeError):
        oracle.gemm(np.zeros((3, 2), np.uint8), np.zeros((2, 2), np.uint8), BF16)
    with pytest.raises(RuntimeError):
        oracle.gemm_rows(np.zeros((3, 2), np.uint16), np.zeros((2, 2), np.uint16), [3], BF16)


def test_tolerance_formula(oracle):
    assert oracle.tolerance(4096, 2.0, 0.5, BF16) == pytest.approx(1e-2 * 64 * 1.0)
    assert oracle.tolerance(64, 448.0, 448.0, E4M3) == pytest.approx(5e-2 * 8 * 448 * 448)


def test_accumulate_into_c_closed_forms(oracle):
    """C = alpha*A*B + beta*C (Section II-A).  With A = I the product is B, so the result is the
    elementwise alpha*B + beta*C_in, exact on small integers; beta = 0 must not read C_in."""
    n = 48
    gen = np.random.default_rng(11)
    Bv = gen.integers(-8, 9, size=(n, n)).astype(np.float64)
    Cv = gen.integers(-8, 9, size=(n, n)).astype(np.float64)
    I = oracle.encode_bf16(np.eye(n))
    B, Cin = oracle.encode_bf16(Bv), oracle.encode_bf16(Cv)
    _, prod = oracle.gemm(I, B, BF16, alpha=0.5)
    c16, c64 = oracle.accumulate(prod, -2.0, Cin)
    assert np.array_equal(c64, 0.5 * Bv - 2.0 * Cv)
    assert np.array_equal(oracle.decode_bf16(c16), 0.5 * Bv - 2.0 * Cv)
    # beta = 1 on a rank-1 product: u v^T + C
    u = gen.integers(-3, 4, size=(n, 1)).astype(np.float64)
    v = gen.integers(-3, 4, size=(1, n)).astype(np.float64)
    _, prod = oracle.gemm(oracle.encode_bf16(u), oracle.encode_bf16(v), BF16)
    _, c64 = oracle.accumulate(prod, 1.0, Cin)
    assert np.array_equal(c64, u @ v + Cv)
    # beta = 0: NaN in C_in does not propagate and C_in is not even decoded
    nan = np.full((n, n), 0x7FC0, np.uint16)
    c16, c64 = oracle.accumulate(prod, 0.0, nan)
    assert np.array_equal(c64, u @ v) and not np.isnan(oracle.decode_bf16(c16)).any()
    c16, c64 = oracle.accumulate(prod, 1.0, nan)
    assert np.isnan(c64).all()
    with pytest.raises(ValueError):
        oracle.accumulate(prod, 1.0, nan[:4])


FP16 = 2


def test_fp16_codec_every_code_against_numpy_half(oracle):
    """binary16 decode of all 65536 codes and encode of many doubles against numpy's float16,
    an independent implementation of the same IEEE format."""
    codes = np.arange(65536, dtype=np.uint16)
    got = oracle.decode_fp16(codes)
    with np.errstate(invalid="ignore"):
        ref = codes.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))
    # every finite code survives a round trip
    assert np.array_equal(oracle.encode_fp16(got[~nan]), codes[~nan])
    gen = np.random.default_rng(12)
    x = np.concatenate([gen.standard_normal(200000) * 10.0 ** gen.integers(-9, 6, 200000),
                        [0.0, -0.0, 65504.0, 65519.999, 65520.0, 1e9, -1e9, np.inf, -np.inf,
                         2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25]])
    # midpoints between neighbouring codes: ties must go to the even code
    lo = gen.integers(0, 0x7BFF, 20000).astype(np.uint16)
    mids = (oracle.decode_fp16(lo) + oracle.decode_fp16(lo + 1)) / 2.0
    x = np.concatenate([x, mids, -mids])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.encode_fp16(x), ref)
    assert oracle.encode_fp16(np.array([np.nan]))[0] & 0x7C00 == 0x7C00 and oracle.encode_fp16(np.array([np.nan]))[0] & 0x3FF


def test_fp16_gemm_closed_forms_and_literal_loop(oracle):
    n = 40
    gen = np.random.default_rng(13)
    X = gen.integers(-20, 21, size=(n, n)).astype(np.float64) / 8.0       # exact in fp16
    Xh = oracle.encode_fp16(X)
    I = oracle.encode_fp16(np.eye(n))
    c16, c64 = oracle.gemm(I, Xh, FP16)
    assert np.array_equal(c16, Xh) and np.array_equal(c64, X)            # output codes are fp16, not bf16
    P = np.eye(n)[gen.permutation(n)]
    c16, c64 = oracle.gemm(oracle.encode_fp16(P), Xh, FP16, alpha=2.0)
    assert np.array_equal(c64, 2.0 * (P @ X)) and np.array_equal(oracle.decode_fp16(c16), 2.0 * (P @ X))
    u = gen.integers(-6, 7, size=(n, 1)).astype(np.float64)
    v = gen.integers(-6, 7, size=(1, n)).astype(np.float64)
    _, c64 = oracle.gemm(oracle.encode_fp16(u), oracle.encode_fp16(v), FP16)
    assert np.array_equal(c64, u @ v)
    A = gen.standard_normal((17, 33)).astype(np.float16).view(np.uint16)
    B = gen.standard_normal((33, 24)).astype(np.float16).view(np.uint16)
    a16, a64 = oracle.gemm(A, B, FP16, alpha=0.375, literal=True)
    b16, b64 = oracle.gemm(A, B, FP16, alpha=0.375)
    assert np.array_equal(a16, b16) and np.array_equal(a64, b64)
    ref = 0.375 * (A.view(np.float16).astype(np.float64) @ B.view(np.float16).astype(np.float64))
    assert np.max(np.abs(a64 - ref)) <= 1e-12
    r16, r64 = oracle.gemm_rows(A, B, np.array([0, 16]), FP16, alpha=0.375)
    assert np.array_equal(r16, a16[[0, 16]])
    s16, _ = oracle.gemm_samples(A, B, np.array([3, 9]), np.array([5, 23]), FP16, alpha=0.375)
    assert np.array_equal(s16, a16[[3, 9], [5, 23]])
    # a sum that overflows binary16 becomes infinity in the code and stays finite in fp64
    big = oracle.encode_fp16(np.full((1, 8), 200.0))
    c16, c64 = oracle.gemm(big, big.T.copy(), FP16)
    assert c64[0, 0] == 320000.0 and c16[0, 0] == 0x7C00
