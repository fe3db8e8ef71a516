"""GPU parity of the fp16 path (the paper's evaluation precision: fp16 in, fp32 accumulate, fp16 out)."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

pytestmark = pytest.mark.gpu

FP16 = 2


@pytest.fixture(scope="module")
def g():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04226_amd import binding
    return binding


@pytest.mark.parametrize("b_layout", [0, 1])
@pytest.mark.parametrize("shape", [(200, 264, 328), (520, 776, 1024)])
def test_fp16_every_config_bit_exact_on_integers(g, oracle, shape, b_layout):
    """Every variant, split-K factor and Stream-K entry, both storages of B.  Sums stay below 2^11
    in magnitude only by luck, so the check is on codes: the fp32 sum is exact (integers below
    2^24) and both sides round the same exact value to fp16 once."""
    from gpu_util import run_cfg, to_dev
    M, N, K = shape
    A, B = wl.integer_fp16(M, N, K, seed=61, case=M)
    ref16, _ = oracle.gemm(A, B, FP16)
    dA, dB = to_dev(A), to_dev(np.ascontiguousarray(B.T) if b_layout else B)
    n_run, kinds = 0, set()
    for idx in range(g.gemm_cfg_count(FP16)):
        c = g.gemm_cfg_at_ex(idx, M, N, K, FP16, b_layout)
        if c is None:
            continue
        out = run_cfg(c, dA, dB, M, N)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        n_run += 1
        kinds.add("streamk" if c.stream_k else "split" if c.split_k > 1 else "dp")
    assert n_run >= 60 and {"dp", "split"} <= kinds


def test_fp16_square_4096_k_contiguous_within_tolerance(g, oracle):
    """The paper's own configuration: fp16, both operands K-contiguous (Section V)."""
    from gpu_util import run_cfg, to_dev
    n = 4096
    A, B = wl.normal_fp16(n, n, n, seed=62)
    rows = np.unique(np.concatenate([np.arange(0, n, 131), [255, 256, n - 1]]))
    _, ref64 = oracle.gemm_rows(A, B, rows, FP16)
    tol = oracle.tolerance(n, float(np.abs(oracle.decode_fp16(A)).max()), float(np.abs(oracle.decode_fp16(B)).max()), FP16)
    dA = to_dev(A)
    for b_layout in (1, 0):
        dB = to_dev(np.ascontiguousarray(B.T) if b_layout else B)
        c = g.gemm_select_ex(n, n, n, FP16, b_layout)
        out = run_cfg(c, dA, dB, n, n)
        err = np.abs(oracle.decode_fp16(out[rows]) - ref64).max()
        assert err <= tol, (c.describe(), err, tol)


def test_fp16_beta_and_alpha(g, oracle):
    from gpu_util import to_dev, workspace_for
    M, N, K = 300, 520, 1096
    A, B = wl.integer_fp16(M, N, K, seed=63)
    gen = np.random.default_rng(64)
    Cin = oracle.encode_fp16(gen.integers(-32, 33, size=(M, N)).astype(np.float64))
    _, prod = oracle.gemm(A, B, FP16, alpha=0.25)
    ref16, _ = oracle.accumulate(prod, 2.0, Cin, FP16)
    dA, dB = to_dev(A), to_dev(B)
    seen = set()
    for idx in range(g.gemm_cfg_count(FP16)):
        c = g.gemm_cfg_at(idx, M, N, K, FP16)
        if c is None or c.split_k > 2:
            continue
        c.alpha, c.beta = 0.25, 2.0
        workspace_for(c)
        dC = to_dev(Cin).clone()
        g.gemm_run(c, dA, dB, dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        seen.add("streamk" if c.stream_k else "split" if c.split_k > 1 else "dp")
    assert {"dp", "split"} <= seen
