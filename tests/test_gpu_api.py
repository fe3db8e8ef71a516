"""The one-call convenience (`api.matmul`) against the CPU oracle: it only picks the cfg, keeps the
workspace and forwards to gemm_run, so a few shapes that exercise those steps are enough."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_matmul_matches_the_oracle_across_dtypes_layouts_and_strides(oracle):
    from paper_2512_04226_amd import api, binding as g
    from gpu_util import to_dev
    # bf16, a shape whose pick splits K (workspace path), then a plain one; integer data: bit-exact
    for (M, N, K) in [(64, 64, 16384), (300, 520, 72), (1024, 1032, 512)]:
        A, B = wl.integer_bf16(M, N, K, seed=91)
        ref16, _ = oracle.gemm(A, B, oracle.BF16)
        dA, dB = to_dev(A).view(torch.bfloat16), to_dev(B).view(torch.bfloat16)
        C = api.matmul(dA, dB)
        torch.cuda.synchronize()
        assert C.dtype == torch.bfloat16 and np.array_equal(C.view(torch.int16).cpu().numpy().view(np.uint16), ref16)
        # the same through the K-contiguous layout and padded leading dimensions
        big = torch.zeros((N, K + 64), dtype=torch.bfloat16, device="cuda")
        big[:, :K] = dB.t()
        out = torch.full((M, N + 8), float("nan"), dtype=torch.bfloat16, device="cuda")
        api.matmul(dA, big[:, :K], out=out[:, :N], b_k_contiguous=True)
        torch.cuda.synchronize()
        assert np.array_equal(out[:, :N].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), ref16)
        assert torch.isnan(out[:, N:]).all()
    assert api.select(64, 64, 16384, g.GEMM_BF16).split_k > 1          # the workspace path was taken
    assert api.select(64, 64, 16384, g.GEMM_BF16) is api.select(64, 64, 16384, g.GEMM_BF16)   # memoised
    # fp16 with alpha and beta (exact on integer data)
    M, N, K = 200, 264, 328
    A, B = wl.integer_fp16(M, N, K, seed=92)
    _, ref64 = oracle.gemm(A, B, oracle.FP16, alpha=0.5)
    cin = wl.f32_to_fp16_bits(np.random.default_rng(93).integers(-8, 9, size=(M, N)).astype(np.float32))
    want, _ = oracle.accumulate(ref64, 2.0, cin, oracle.FP16)
    out = to_dev(cin).view(torch.float16)
    api.matmul(to_dev(A).view(torch.float16), to_dev(B).view(torch.float16), out=out, alpha=0.5, beta=2.0)
    torch.cuda.synchronize()
    assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), want)
    # fp8: quantised operands, scales through alpha
    if hasattr(torch, "float8_e4m3fn"):
        M, N, K = 256, 512, 1024
        Aq, Bq, sa, sb = wl.normal_e4m3(M, N, K, seed=94)
        alpha = float(np.float32(sa * sb))
        _, ref64 = oracle.gemm(Aq, Bq, oracle.E4M3, alpha=alpha)
        C = api.matmul(to_dev(Aq).view(torch.float8_e4m3fn), to_dev(Bq).view(torch.float8_e4m3fn), alpha=alpha)
        torch.cuda.synchronize()
        got = (C.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        amax = float(np.abs(oracle.decode(Aq, oracle.E4M3)).max() * sa), float(np.abs(oracle.decode(Bq, oracle.E4M3)).max() * sb)
        assert np.max(np.abs(got - ref64)) <= oracle.tolerance(K, amax[0], amax[1], oracle.E4M3)
    with pytest.raises(TypeError):
        api.matmul(dA.float(), dB.float())
    with pytest.raises(ValueError):
        api.matmul(dA, dB[:-8])


@pytest.mark.parametrize("shape", [(1, 8, 8), (7, 8, 65536), (65537, 8, 8), (300001, 64, 64), (3, 16400, 24), (2049, 8, 4104)])
def test_extreme_aspect_ratios_bit_exact(oracle, shape):
    """Shapes at the edges of what the tiles were made for: one row, one 8-wide column block, a very
    tall or very deep problem.  Integer data: exactly one correct result."""
    from paper_2512_04226_amd import api
    from gpu_util import to_dev
    M, N, K = shape
    A, B = wl.integer_bf16(M, N, K, seed=95)
    ref16, _ = oracle.gemm(A, B, oracle.BF16)
    C = api.matmul(to_dev(A).view(torch.bfloat16), to_dev(B).view(torch.bfloat16))
    torch.cuda.synchronize()
    got = C.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, ref16), (shape, api.select(M, N, K, 0).describe(), int((got != ref16).sum()))
