"""gemm_run_noalloc (the entry point for callers that cannot allocate) against gemm_run, through the
C ABI: same cfg, same operands, bit-identical C, on two calls in a row of which the second is smaller
(so it runs on a buffer that still holds the first call's partial sums)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _cfgs(g, M, N, K, dtype):
    """One split-K and one Stream-K configuration for the shape that fit the built-in buffer, plus the
    plain pick."""
    out = {}
    for idx in range(g.gemm_cfg_count(dtype)):
        c = g.gemm_cfg_at(idx, M, N, K, dtype)
        if c is None or g.gemm_workspace_bytes(c) > g.GEMM_NOALLOC_WORKSPACE_BYTES:
            continue
        if c.stream_k and "stream_k" not in out:
            out["stream_k"] = c
        if c.split_k == 4 and c.block_m <= 128 and "split_k" not in out:
            out["split_k"] = c
    out["pick"] = g.gemm_select(M, N, K, dtype)
    return out


def test_noalloc_matches_gemm_run_on_two_calls_in_a_row():
    from paper_2512_04226_amd import binding as g
    from paper_2512_04226_amd import workloads as wl
    from tests.gpu_util import to_dev

    ws = None
    try:
        ran = set()
        for (M, N, K) in ((520, 776, 2048), (200, 264, 1024)):      # the second call is the smaller one
            A, B = wl.integer_bf16(M, N, K, seed=7, case=M)
            dA, dB = to_dev(A), to_dev(B)
            for kind, cfg in _cfgs(g, M, N, K, g.GEMM_BF16).items():
                need = g.gemm_workspace_bytes(cfg)
                if need and (ws is None or ws.numel() * 4 < need):
                    ws = torch.empty((need + 3) // 4, dtype=torch.float32, device="cuda")
                if ws is not None:
                    g.gemm_set_workspace(ws)
                want = torch.full((M, N), 0x7FC0, dtype=torch.int16, device="cuda")
                g.gemm_run(cfg, dA, dB, want)
                torch.cuda.synchronize()
                g.gemm_set_workspace(None)            # the new entry point must not depend on a registered buffer
                got = torch.full((M, N), 0x7FC0, dtype=torch.int16, device="cuda")
                g.gemm_run_noalloc(cfg, dA, dB, got)
                torch.cuda.synchronize()
                assert torch.equal(got, want), (kind, cfg.describe())
                ran.add(kind)
        assert {"split_k", "stream_k", "pick"} <= ran, ran
    finally:
        g.gemm_set_workspace(None)


def test_noalloc_matches_the_oracle_and_refuses_what_does_not_fit(oracle):
    from paper_2512_04226_amd import binding as g
    from paper_2512_04226_amd import workloads as wl
    from tests.gpu_util import to_dev

    M, N, K = 72, 1032, 4096
    A, B = wl.integer_bf16(M, N, K, seed=7, case=1)
    cfg = next(c for c in (g.gemm_cfg_at(i, M, N, K, g.GEMM_BF16) for i in range(g.gemm_cfg_count(g.GEMM_BF16)))
               if c is not None and c.split_k == 8)
    dC = torch.full((M, N), 0x7FC0, dtype=torch.int16, device="cuda")
    g.gemm_run_noalloc(cfg, to_dev(A), to_dev(B), dC)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().view(np.uint16), oracle.gemm(A, B, oracle.BF16)[0])
    # a split-K cfg whose slabs need more than the built-in buffer (136 MiB here): refused, nothing launched
    big = next(c for c in (g.gemm_cfg_at(i, 4352, 4096, 4096, g.GEMM_BF16) for i in range(g.gemm_cfg_count(g.GEMM_BF16)))
               if c is not None and g.gemm_workspace_bytes(c) > g.GEMM_NOALLOC_WORKSPACE_BYTES)
    dA = torch.zeros((4352, 4096), dtype=torch.int16, device="cuda")
    dB = torch.zeros((4096, 4096), dtype=torch.int16, device="cuda")
    dC = torch.full((4352, 4096), 0x7FC0, dtype=torch.int16, device="cuda")
    with pytest.raises(g.GemmError) as e:
        g.gemm_run_noalloc(big, dA, dB, dC)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert bool((dC == 0x7FC0).all())
