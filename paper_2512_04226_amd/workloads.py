"""Seeded synthetic inputs for the GEMM workloads (no GEMM arithmetic lives here).

The paper evaluates on random FP16 problem shapes (Section V-A) and on matrix sizes
derived from Llama 3 whose values it does not list (Section V-D).  These generators
stand in for both: fixed-seed numpy draws, converted to the bit patterns that both the
GPU library and the CPU checker consume.  bf16 travels as uint16, fp8 e4m3 as uint8.

Every generator is a pure function of its arguments (PCG64 seeded by [seed, case]).
"""
import math

import numpy as np

BF16 = 0
E4M3 = 1


def f32_to_bf16_bits(x):
    """float32 -> bf16 bit patterns, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize_e4m3(x):
    """Per-tensor scaled cast to fp8 e4m3: scale = max|x| / 448, codes = cast(x / scale).

    Returns (uint8 codes, float32 scale).  After scaling nothing exceeds 448, so the
    cast never overflows.  The cast itself is torch's CPU float8_e4m3fn conversion.
    """
    import torch

    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = float(np.max(np.abs(x))) if x.size else 0.0
    scale = np.float32(amax / 448.0) if amax > 0 else np.float32(1.0)
    scaled = torch.from_numpy(x / scale).clamp_(-448.0, 448.0)
    codes = scaled.to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()
    return codes, scale


def _rng(seed, case=0):
    return np.random.default_rng([seed, case])


def uniform_bf16(M, N, K, seed, case=0):
    """A (MxK) and B (KxN) uniform in [-1, 1], as bf16 bits."""
    g = _rng(seed, case)
    A = g.uniform(-1.0, 1.0, size=(M, K)).astype(np.float32)
    B = g.uniform(-1.0, 1.0, size=(K, N)).astype(np.float32)
    return f32_to_bf16_bits(A), f32_to_bf16_bits(B)


def f32_to_fp16_bits(x):
    """float32 -> IEEE binary16 bit patterns (numpy's round-to-nearest-even cast)."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def integer_fp16(M, N, K, seed, case=0, lo=-4, hi=4):
    """Integer-valued operands in [lo, hi] as fp16 bits (exactly representable)."""
    g = _rng(seed, case)
    A = g.integers(lo, hi + 1, size=(M, K)).astype(np.float32)
    B = g.integers(lo, hi + 1, size=(K, N)).astype(np.float32)
    return f32_to_fp16_bits(A), f32_to_fp16_bits(B)


def normal_fp16(M, N, K, seed, case=0, std_a=1.0, std_b=1.0):
    """A ~ N(0, std_a), B ~ N(0, std_b) as fp16 bits: the paper's evaluation precision (Section V),
    with the value distribution of the square bf16 workload."""
    g = _rng(seed, case)
    A = g.standard_normal(size=(M, K), dtype=np.float32) * np.float32(std_a)
    B = g.standard_normal(size=(K, N), dtype=np.float32) * np.float32(std_b)
    return f32_to_fp16_bits(A), f32_to_fp16_bits(B)


def integer_bf16(M, N, K, seed, case=0, lo=-4, hi=4):
    """Integer-valued operands in [lo, hi] (exactly representable in bf16)."""
    g = _rng(seed, case)
    A = g.integers(lo, hi + 1, size=(M, K)).astype(np.float32)
    B = g.integers(lo, hi + 1, size=(K, N)).astype(np.float32)
    return f32_to_bf16_bits(A), f32_to_bf16_bits(B)


def normal_bf16(M, N, K, seed, case=0, std_a=1.0, std_b=1.0):
    """A ~ N(0, std_a), B ~ N(0, std_b) as bf16 bits (drawn in float32, row blocks)."""
    g = _rng(seed, case)
    A = (g.standard_normal(size=(M, K), dtype=np.float32) * np.float32(std_a))
    B = np.empty((K, N), np.uint16)
    step = max(1, (1 << 24) // max(N, 1))
    for r in range(0, K, step):
        blk = g.standard_normal(size=(min(step, K - r), N), dtype=np.float32) * np.float32(std_b)
        B[r:r + blk.shape[0]] = f32_to_bf16_bits(blk)
    return f32_to_bf16_bits(A), B


def normal_e4m3(M, N, K, seed, case=0):
    """A, B ~ N(0,1), each scaled so max|x| = 448 and cast to e4m3.

    Returns (A_codes, B_codes, scale_a, scale_b); the real-valued product is
    (scale_a * scale_b) * (A_codes . B_codes).
    """
    g = _rng(seed, case)
    A = g.standard_normal(size=(M, K), dtype=np.float32)
    B = g.standard_normal(size=(K, N), dtype=np.float32)
    Aq, sa = quantize_e4m3(A)
    Bq, sb = quantize_e4m3(B)
    return Aq, Bq, sa, sb


# ---- the five benchmark configurations ----

def config1(integer=False):
    """512^3, uniform [-1,1] from seed 0 (or integers in [-4,4], same seed, case 1)."""
    if integer:
        return integer_bf16(512, 512, 512, seed=0, case=1)
    return uniform_bf16(512, 512, 512, seed=0, case=0)


def config2(n=4096):
    """Square bf16 GEMM (n = 4096 or 8192), N(0,1), seed 1."""
    return normal_bf16(n, n, n, seed=1, case=n)


SKINNY_M = (1, 16, 64, 256)
SKINNY_NK = ((28672, 8192), (8192, 28672))


def config3(M, N, K):
    """LLM-shaped skinny GEMM: activations N(0,1), weights N(0, 0.02), seed 2."""
    return normal_bf16(M, N, K, seed=2, case=M * 4 + (0 if N > K else 1), std_a=1.0, std_b=0.02)


def config4(n=8192):
    """fp8 e4m3 square GEMM with per-tensor scales, seed 3."""
    return normal_e4m3(n, n, n, seed=3, case=n)


def config5_shapes(count=64, seed=4, lo=64, hi=16384):
    """Irregular shapes: each of M, N, K log-uniform in [lo, hi], rounded to a multiple of 16."""
    g = np.random.default_rng(seed)
    u = g.uniform(math.log(lo), math.log(hi), size=(count, 3))
    dims = 16 * np.rint(np.exp(u) / 16.0).astype(np.int64)
    dims = np.clip(dims, lo, hi)
    return [tuple(int(v) for v in row) for row in dims]


def uniform128_shapes(count=192, seed=5, hi=8192):
    """Shapes drawn like those of the paper's selection-efficiency experiment (Section V-A): each of
    M, N, K a uniformly random multiple of 128 up to 8192.  The paper uses 150,000 of them; this is a
    seeded sample."""
    g = np.random.default_rng(seed)
    dims = 128 * g.integers(1, hi // 128 + 1, size=(count, 3))
    return [tuple(int(v) for v in row) for row in dims]


def config5(index, shapes=None):
    shapes = shapes or config5_shapes()
    M, N, K = shapes[index]
    return uniform_bf16(M, N, K, seed=4, case=index + 1)


def routed_rows(groups, total_rows, seed, skew=1.0):
    """Rows per group of a grouped launch shaped like expert routing: Dirichlet(skew) shares of
    total_rows, multinomial counts -- ragged, and a group may get no row at all."""
    rng = _rng(seed, groups)
    shares = rng.dirichlet(np.full(groups, skew))
    return [int(x) for x in rng.multinomial(total_rows, shares)]
