"""Shapes whose N or K is not a whole number of 16-byte chunks (the boundary takes every M, N, K >= 1;
only pointers and leading dimensions must be 16-byte aligned).  Integer-valued operands, so every
configuration must reproduce the oracle bit for bit; the padding between N (or K) and the leading
dimension holds NaN patterns that must not leak into the result, and C's padding must stay untouched."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

pytestmark = pytest.mark.gpu

BF16, E4M3, FP16 = 0, 1, 2
POISON16 = 0x7FC0


def _up(x, m):
    return -(-x // m) * m


def _padded(bits, ld, fill):
    out = np.full((bits.shape[0], ld), fill, bits.dtype)
    out[:, :bits.shape[1]] = bits
    return out


def _operands(oracle, M, N, K, dtype, seed):
    if dtype == E4M3:
        gen = np.random.default_rng([seed, M, N, K])
        vals = np.array([0, 1, 2, 3, 4, -1, -2, -3, -4], dtype=np.float64)
        return (oracle.encode_e4m3(vals[gen.integers(0, 9, size=(M, K))]),
                oracle.encode_e4m3(vals[gen.integers(0, 9, size=(K, N))]))
    return wl.integer_bf16(M, N, K, seed=seed, case=M + 3 * N + 7 * K)


def _run_all(g, oracle, M, N, K, dtype, b_layout, extra_ld=0):
    from gpu_util import to_dev, workspace_for
    per16 = 16 if dtype == E4M3 else 8
    nan_in = 0x7F if dtype == E4M3 else POISON16
    A, B = _operands(oracle, M, N, K, dtype, seed=11)
    ref16, _ = oracle.gemm(A, B, dtype)
    lda = _up(K, per16) + extra_ld * per16
    Bs = np.ascontiguousarray(B.T) if b_layout else B
    ldb = _up(Bs.shape[1], per16) + extra_ld * per16
    ldc = _up(N, 8) + extra_ld * 8
    dA, dB = to_dev(_padded(A, lda, nan_in)), to_dev(_padded(Bs, ldb, nan_in))
    n_run = kinds = 0
    seen = set()
    for idx in range(g.gemm_cfg_count(dtype)):
        c = g.gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout)
        if c is None:
            continue
        assert (c.lda, c.ldb, c.ldc) == (_up(K, per16), _up(Bs.shape[1], per16), _up(N, 8))   # the smallest legal ones
        c.lda, c.ldb, c.ldc = lda, ldb, ldc
        workspace_for(c)
        dC = torch.full((M, ldc), POISON16, dtype=torch.int16, device="cuda")
        g.gemm_run(c, dA, dB, dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16)
        assert np.array_equal(out[:, :N], ref16), (c.describe(), int((out[:, :N] != ref16).sum()))
        assert (out[:, N:] == POISON16).all(), (c.describe(), "C's padding was written")
        n_run += 1
        seen.add("stream_k" if c.stream_k else "split" if c.split_k > 1 else "plain")
    return n_run, seen


@pytest.fixture(scope="module")
def g():
    from paper_2512_04226_amd import binding
    return binding


@pytest.mark.parametrize("shape", [(5, 1, 7), (33, 1001, 72), (64, 64, 4097), (1, 9, 1), (130, 258, 515)])
@pytest.mark.parametrize("b_layout", [0, 1])
def test_ragged_bf16_every_configuration_bit_exact(g, oracle, shape, b_layout):
    M, N, K = shape
    n_run, seen = _run_all(g, oracle, M, N, K, BF16, b_layout, extra_ld=1 if M > 5 else 0)
    assert n_run >= 30 and "plain" in seen
    if K >= 512:
        assert "split" in seen


@pytest.mark.parametrize("shape", [(17, 24, 40), (5, 1, 7), (70, 130, 1000)])
@pytest.mark.parametrize("b_layout", [0, 1])
def test_ragged_fp8_every_configuration_bit_exact(g, oracle, shape, b_layout):
    M, N, K = shape
    n_run, _ = _run_all(g, oracle, M, N, K, E4M3, b_layout, extra_ld=1)
    assert n_run >= 15


def test_ragged_stream_k_and_fp16(g, oracle):
    """A ragged shape with a partial last wave of tiles (Stream-K candidates exist), and the fp16 instantiations."""
    n_run, seen = _run_all(g, oracle, 520, 777, 1027, BF16, 0)
    assert "stream_k" in seen and "split" in seen
    from gpu_util import to_dev
    M, N, K = 45, 100, 99
    A, B = wl.integer_fp16(M, N, K, seed=5, case=1)
    ref16, _ = oracle.gemm(A, B, FP16)
    dA, dB = to_dev(_padded(A, _up(K, 8), 0x7E00)), to_dev(_padded(B, _up(N, 8), 0x7E00))
    c = g.gemm_select(M, N, K, FP16)
    dC = torch.full((M, c.ldc), 0x7E00, dtype=torch.int16, device="cuda")
    g.gemm_run(c, dA, dB, dC)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().view(np.uint16)
    assert np.array_equal(out[:, :N], ref16) and (out[:, N:] == 0x7E00).all()


def test_ragged_beta_and_random_data_through_matmul(g, oracle):
    """C = alpha*A*B + beta*C on a ragged shape (integer data, power-of-two scalars: exact), and api.matmul on
    views with odd extents of N(0,1) data within the benchmark's tolerance."""
    from gpu_util import bf16_to_f64, to_dev
    from paper_2512_04226_amd import api
    M, N, K = 37, 61, 203
    A, B = wl.integer_bf16(M, N, K, seed=3, case=9)
    Cin = wl.integer_bf16(M, N, 8, seed=4, case=9)[0][:, :1].repeat(N, axis=1)      # small integers as bf16 bits
    _, prod = oracle.gemm(A, B, BF16, alpha=0.5)
    ref16, _ = oracle.accumulate(prod, 2.0, Cin)
    for c in (g.gemm_select(M, N, K, BF16),
              next(x for x in (g.gemm_cfg_at(i, M, N, K, BF16) for i in range(g.gemm_cfg_count(BF16)))
                   if x is not None and x.split_k == 2)):
        from gpu_util import workspace_for
        workspace_for(c)
        c.alpha, c.beta = 0.5, 2.0
        dC = to_dev(_padded(Cin, c.ldc, POISON16))
        g.gemm_run(c, to_dev(_padded(A, c.lda, POISON16)), to_dev(_padded(B, c.ldb, POISON16)), dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16)
        assert np.array_equal(out[:, :N], ref16) and (out[:, N:] == POISON16).all(), c.describe()
    gen = torch.Generator(device="cuda").manual_seed(5)
    Af = torch.randn((300, 1096), device="cuda", generator=gen).to(torch.bfloat16)
    Bf = torch.randn((1096, 520), device="cuda", generator=gen).to(torch.bfloat16)
    Av, Bv = Af[:299, :1091], Bf[:1091, :517]          # odd extents, 16-byte aligned rows
    out = api.matmul(Av, Bv)
    assert out.shape == (299, 517)
    An = Av.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    Bn = Bv.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    _, ref64 = oracle.gemm(An, Bn, BF16)
    got = bf16_to_f64(out.view(torch.int16).cpu().numpy().view(np.uint16))
    tol = oracle.tolerance(1091, float(Av.abs().max()), float(Bv.abs().max()), BF16)
    assert float(np.max(np.abs(got - ref64))) <= tol
