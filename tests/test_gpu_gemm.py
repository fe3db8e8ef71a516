"""GPU parity: the HIP kernels (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1


@pytest.fixture(scope="module")
def g():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04226_amd import binding
    return binding


def _all_cfgs(g, M, N, K, dtype):
    out = []
    for idx in range(g.gemm_cfg_count(dtype)):
        c = g.gemm_cfg_at(idx, M, N, K, dtype)
        if c is not None:
            out.append((idx, c))
    return out


@pytest.mark.parametrize("shape", [(200, 264, 328), (512, 512, 512)])
def test_bf16_every_variant_bit_exact_on_integers(g, oracle, shape):
    """Integer operands in [-4,4], K <= 512: every partial sum is an integer below 2^24, so
    any fp32 summation order is exact and the bf16 result is unique."""
    from gpu_util import run_cfg, to_dev
    M, N, K = shape
    A, B = wl.integer_bf16(M, N, K, seed=0, case=1)
    ref16, _ = oracle.gemm(A, B, BF16)
    dA, dB = to_dev(A), to_dev(B)
    cfgs = _all_cfgs(g, M, N, K, BF16)
    assert len(cfgs) > 50
    bad = []
    for idx, c in cfgs:
        out = run_cfg(c, dA, dB, M, N)
        if not np.array_equal(out, ref16):
            bad.append((idx, c.describe(), int((out != ref16).sum())))
    assert not bad, bad[:10]


@pytest.mark.parametrize("shape", [(200, 272, 336), (256, 256, 512)])
def test_fp8_every_variant_bit_exact_on_integers(g, oracle, shape):
    from gpu_util import run_cfg, to_dev
    M, N, K = shape
    gen = np.random.default_rng(3)
    vals = np.array([0, 1, 2, 3, 4, -1, -2, -3, -4], dtype=np.float64)
    A = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(M, K))])
    B = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(K, N))])
    ref16, _ = oracle.gemm(A, B, E4M3, alpha=0.5)
    dA, dB = to_dev(A), to_dev(B)
    bad = []
    for idx, c in _all_cfgs(g, M, N, K, E4M3):
        out = run_cfg(c, dA, dB, M, N, alpha=0.5)
        if not np.array_equal(out, ref16):
            bad.append((idx, c.describe(), int((out != ref16).sum())))
    assert not bad, bad[:10]


def test_config1_uniform_within_tolerance(g, oracle):
    from gpu_util import bf16_to_f64, run_cfg, to_dev
    A, B = wl.config1()
    _, ref64 = oracle.gemm(A, B, BF16)
    tol = oracle.tolerance(512, 1.0, 1.0, BF16)
    c = g.gemm_select(512, 512, 512, BF16)
    out = run_cfg(c, to_dev(A), to_dev(B), 512, 512)
    err = np.max(np.abs(bf16_to_f64(out) - ref64))
    assert err <= tol, (err, tol, c.describe())
    # bf16 rounding of an fp32 sum should in fact sit within a few output ulps
    assert err <= 2.0 ** -7 * np.abs(ref64).max()
