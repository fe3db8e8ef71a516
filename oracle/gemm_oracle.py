"""ctypes front end of the CPU GEMM oracle (TEST INFRASTRUCTURE ONLY).

Wraps oracle/gemm_oracle.c: Algorithm 1 of the paper (Section II-A) in fp64 with the
result rounded once to the 16-bit output format (bf16; fp16 for fp16 inputs).  Nothing under the product package imports this module;
it is for tests, the smoke check and the bench's cpu_baseline leg.

Arrays are numpy: bf16 and fp16 as uint16 bit patterns, e4m3 as uint8 bit patterns.
"""
import ctypes
import os
import subprocess

import numpy as np

BF16 = 0
E4M3 = 1
FP16 = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (host only, no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".%d.tmp" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    i64, dbl, vp, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
    for name in ("oracle_gemm", "oracle_gemm_alg1"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, dbl, vp, i64, vp]
    lib.oracle_gemm_rows.restype = ci
    lib.oracle_gemm_rows.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, dbl, i64, vp, vp, vp]
    lib.oracle_gemm_samples.restype = ci
    lib.oracle_gemm_samples.argtypes = [i64, i64, i64, vp, i64, vp, i64, ci, dbl, i64, vp, vp, vp, vp]
    for name in ("oracle_decode_bf16", "oracle_decode_e4m3", "oracle_encode_bf16", "oracle_encode_e4m3",
                 "oracle_decode_fp16", "oracle_encode_fp16"):
        f = getattr(lib, name)
        f.restype = None
        f.argtypes = [i64, vp, vp]
    _lib = lib
    return lib


def _in_dtype(dtype):
    if dtype in (BF16, FP16):
        return np.uint16
    if dtype == E4M3:
        return np.uint8
    raise ValueError("dtype must be BF16 (0), E4M3 (1) or FP16 (2)")


def _check_operands(A, B, dtype):
    t = _in_dtype(dtype)
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    if A.dtype != t or B.dtype != t:
        raise TypeError("operands must be %s bit patterns" % np.dtype(t).name)
    if A.ndim != 2 or B.ndim != 2 or A.shape[1] != B.shape[0]:
        raise ValueError("A must be MxK and B KxN")
    return A, B


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def gemm(A, B, dtype=BF16, alpha=1.0, literal=False):
    """Full product.  Returns (C_bf16_bits uint16 MxN, C_f64 MxN).

    literal=True runs the i/j/reduction loop nest exactly as Algorithm 1 prints it
    (single thread); the default walks B by rows with the same per-element sums.
    """
    A, B = _check_operands(A, B, dtype)
    M, K = A.shape
    N = B.shape[1]
    C16 = np.empty((M, N), np.uint16)
    C64 = np.empty((M, N), np.float64)
    fn = _load().oracle_gemm_alg1 if literal else _load().oracle_gemm
    rc = fn(M, N, K, _ptr(A), K, _ptr(B), N, dtype, float(alpha), _ptr(C16), N, _ptr(C64))
    if rc != 0:
        raise RuntimeError("oracle_gemm failed: %d" % rc)
    return C16, C64


def gemm_rows(A, B, rows, dtype=BF16, alpha=1.0):
    """Rows `rows` of the product: (bf16 bits, fp64), each len(rows) x N."""
    A, B = _check_operands(A, B, dtype)
    M, K = A.shape
    N = B.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    C16 = np.empty((len(rows), N), np.uint16)
    C64 = np.empty((len(rows), N), np.float64)
    rc = _load().oracle_gemm_rows(M, N, K, _ptr(A), K, _ptr(B), N, dtype, float(alpha), len(rows),
                                  _ptr(rows), _ptr(C16), _ptr(C64))
    if rc != 0:
        raise RuntimeError("oracle_gemm_rows failed: %d" % rc)
    return C16, C64


def gemm_samples(A, B, rows, cols, dtype=BF16, alpha=1.0):
    """Elements (rows[s], cols[s]) of the product: (bf16 bits, fp64), each of length n."""
    A, B = _check_operands(A, B, dtype)
    M, K = A.shape
    N = B.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    if rows.shape != cols.shape or rows.ndim != 1:
        raise ValueError("rows and cols must be 1-D and of equal length")
    C16 = np.empty(len(rows), np.uint16)
    C64 = np.empty(len(rows), np.float64)
    rc = _load().oracle_gemm_samples(M, N, K, _ptr(A), K, _ptr(B), N, dtype, float(alpha), len(rows),
                                     _ptr(rows), _ptr(cols), _ptr(C16), _ptr(C64))
    if rc != 0:
        raise RuntimeError("oracle_gemm_samples failed: %d" % rc)
    return C16, C64


def gemm_batched(A, B, dtype=BF16, alpha=1.0):
    """`batch` independent products: A is batch x M x K, B is batch x K x N.  Each problem is one
    call of gemm(); returns (16-bit codes batch x M x N, fp64 batch x M x N)."""
    if A.ndim != 3 or B.ndim != 3 or A.shape[0] != B.shape[0]:
        raise ValueError("A must be batch x M x K and B batch x K x N")
    outs = [gemm(A[b], B[b], dtype, alpha) for b in range(A.shape[0])]
    return np.stack([o[0] for o in outs]), np.stack([o[1] for o in outs])


def gemm_grouped(problems, dtype=BF16, alpha=1.0):
    """Grouped product: problems = [(A_g, B_g), ...] of different shapes, each C_g = alpha * A_g * B_g by
    the plain definition (one gemm() per group; an A with no rows gives an empty result).
    Returns a list of (bits, fp64) pairs."""
    out = []
    for A, B in problems:
        if A.shape[0] == 0:
            out.append((np.zeros((0, B.shape[1]), dtype=np.uint16), np.zeros((0, B.shape[1]))))
        else:
            out.append(gemm(A, B, dtype, alpha))
    return out


def accumulate(C64, beta, C_in_bits, dtype=BF16):
    """The full definition of Section II-A, C = alpha*A*B + beta*C: C64 is the fp64 value of
    alpha*A*B (from gemm / gemm_rows / gemm_samples), C_in_bits the 16-bit codes C held on
    entry (same shape; fp16 when dtype is FP16, else bf16).  Returns (16-bit codes, fp64).  beta == 0 drops the term without reading
    C_in (the BLAS convention: whatever C held, NaN included, does not propagate)."""
    C64 = np.asarray(C64, dtype=np.float64)
    if beta == 0.0:
        out = C64.copy()
    else:
        c_in = decode_out(C_in_bits, dtype)
        if c_in.shape != C64.shape:
            raise ValueError("C_in must have the shape of the product")
        out = C64 + float(beta) * c_in
    return (encode_fp16(out) if dtype == FP16 else encode_bf16(out)), out


def decode_bf16(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, np.float64)
    _load().oracle_decode_bf16(bits.size, _ptr(bits), _ptr(out))
    return out


def decode_e4m3(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    out = np.empty(bits.shape, np.float64)
    _load().oracle_decode_e4m3(bits.size, _ptr(bits), _ptr(out))
    return out


def decode_fp16(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, np.float64)
    _load().oracle_decode_fp16(bits.size, _ptr(bits), _ptr(out))
    return out


def encode_fp16(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, np.uint16)
    _load().oracle_encode_fp16(x.size, _ptr(x), _ptr(out))
    return out


def decode(bits, dtype):
    return {BF16: decode_bf16, E4M3: decode_e4m3, FP16: decode_fp16}[dtype](bits)


def decode_out(bits, dtype):
    """Value of 16-bit output codes: fp16 for fp16 inputs, bf16 otherwise."""
    return decode_fp16(bits) if dtype == FP16 else decode_bf16(bits)


def encode_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, np.uint16)
    _load().oracle_encode_bf16(x.size, _ptr(x), _ptr(out))
    return out


def encode_e4m3(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, np.uint8)
    _load().oracle_encode_e4m3(x.size, _ptr(x), _ptr(out))
    return out


def tolerance(K, max_abs_a, max_abs_b, dtype=BF16):
    """Acceptance bound on max|C - C_ref| for random data: 1e-2 (bf16), 5e-2 (e4m3) or 2e-3
    (fp16: the output carries 11 significant bits against bf16's 8, so the bf16 bound shrinks by
    2^3, rounded up) times sqrt(K) * max|A| * max|B|, with the maxima taken on the real-valued
    operands."""
    factor = {BF16: 1e-2, E4M3: 5e-2, FP16: 2e-3}[dtype]
    return factor * np.sqrt(float(K)) * float(max_abs_a) * float(max_abs_b)
