"""GPU parity of strided-batched runs against the CPU oracle (one oracle GEMM per problem)."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

pytestmark = pytest.mark.gpu

BF16, E4M3, FP16 = 0, 1, 2


@pytest.fixture(scope="module")
def g():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04226_amd import binding
    return binding


def _int_batch(batch, M, N, K, seed, fp16=False):
    gen = wl.integer_fp16 if fp16 else wl.integer_bf16
    ab = [gen(M, N, K, seed=seed, case=b) for b in range(batch)]
    return np.stack([a for a, _ in ab]), np.stack([b for _, b in ab])


@pytest.mark.parametrize("shape", [(5, 200, 264, 328), (3, 520, 776, 1024)])
def test_batched_every_config_bit_exact_dense_strides(g, oracle, shape):
    from gpu_util import to_dev, workspace_for
    batch, M, N, K = shape
    A, B = _int_batch(batch, M, N, K, seed=71)
    ref16, _ = oracle.gemm_batched(A, B, BF16)
    dA, dB = to_dev(A.reshape(batch * M, K)), to_dev(B.reshape(batch * K, N))
    n_run, kinds = 0, set()
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at_batched(idx, M, N, K, batch, BF16)
        if c is None:
            continue
        assert not c.stream_k
        workspace_for(c)
        dC = torch.full((batch * M, N), 0x7FC0, dtype=torch.int16, device="cuda")
        g.gemm_run(c, dA, dB, dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16).reshape(batch, M, N)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        n_run += 1
        kinds.add("split" if c.split_k > 1 else "dp")
    assert n_run >= 60 and kinds == {"dp", "split"}


def test_batched_padded_strides_k_contiguous_b_beta_fp16(g, oracle):
    """Everything at once: fp16, B stored N x K, gaps between the problems (filled with NaN
    codes that must never be read as data nor overwritten), alpha and beta."""
    from gpu_util import to_dev, workspace_for
    batch, M, N, K = 4, 136, 264, 520
    A, B = _int_batch(batch, M, N, K, seed=72, fp16=True)
    gen = np.random.default_rng(73)
    Cin = oracle.encode_fp16(gen.integers(-16, 17, size=(batch, M, N)).astype(np.float64))
    _, prod = oracle.gemm_batched(A, B, FP16, alpha=0.5)
    ref16 = np.stack([oracle.accumulate(prod[b], 2.0, Cin[b], FP16)[0] for b in range(batch)])
    sa, sb, sc = M * K + 64, N * K + 128, M * N + 8
    NAN = 0x7E00
    Af = np.full(batch * sa, NAN, np.uint16)
    Bf = np.full(batch * sb, NAN, np.uint16)
    Cf = np.full(batch * sc, 0x1234, np.uint16)
    for b in range(batch):
        Af[b * sa:b * sa + M * K] = A[b].ravel()
        Bf[b * sb:b * sb + N * K] = np.ascontiguousarray(B[b].T).ravel()
        Cf[b * sc:b * sc + M * N] = Cin[b].ravel()
    dA, dB = to_dev(Af), to_dev(Bf)
    seen = set()
    for idx in range(g.gemm_cfg_count(FP16)):
        c = g.gemm_cfg_at_batched(idx, M, N, K, batch, FP16, g.GEMM_B_K_CONTIGUOUS)
        if c is None or c.split_k > 2:
            continue
        c.stride_a, c.stride_b, c.stride_c, c.alpha, c.beta = sa, sb, sc, 0.5, 2.0
        workspace_for(c)
        dC = to_dev(Cf).clone()
        g.gemm_run(c, dA, dB, dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16)
        for b in range(batch):
            got = out[b * sc:b * sc + M * N].reshape(M, N)
            assert np.array_equal(got, ref16[b]), (c.describe(), b, int((got != ref16[b]).sum()))
            assert np.all(out[b * sc + M * N:(b + 1) * sc] == 0x1234)
        seen.add("split" if c.split_k > 1 else "dp")
    assert seen == {"dp", "split"}


def test_batched_random_selected_cfg_within_tolerance_and_argument_errors(g, oracle):
    from gpu_util import bf16_to_f64, to_dev, workspace_for
    batch, M, N, K = 16, 512, 512, 2048
    ab = [wl.normal_bf16(M, N, K, seed=74, case=b) for b in range(batch)]
    A, B = np.stack([a for a, _ in ab]), np.stack([b for _, b in ab])
    c = g.gemm_select_batched(M, N, K, batch, BF16)
    workspace_for(c)
    dA, dB = to_dev(A.reshape(batch * M, K)), to_dev(B.reshape(batch * K, N))
    dC = torch.full((batch * M, N), 0x7FC0, dtype=torch.int16, device="cuda")
    g.gemm_run(c, dA, dB, dC)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().view(np.uint16).reshape(batch, M, N)
    tol = oracle.tolerance(K, float(np.abs(bf16_to_f64(A)).max()), float(np.abs(bf16_to_f64(B)).max()), BF16)
    for b in (0, 7, 15):
        _, ref64 = oracle.gemm(A[b], B[b], BF16)
        assert np.abs(bf16_to_f64(out[b]) - ref64).max() <= tol, (c.describe(), b)
    bad = c.copy(); bad.stride_c = M * N - 8           # problems would overlap
    with pytest.raises(g.GemmError):
        g.gemm_run(bad, dA, dB, dC)
    bad = c.copy(); bad.stride_a = M * K + 4           # breaks the 16-byte alignment
    with pytest.raises(g.GemmError):
        g.gemm_run(bad, dA, dB, dC)
    bad = c.copy(); bad.batch = 0
    with pytest.raises(g.GemmError):
        g.gemm_run(bad, dA, dB, dC)
