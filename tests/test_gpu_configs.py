"""GPU parity at the benchmark configurations' full sizes (through the C ABI, in the launch
configuration the selector picks), on outputs the oracle can compute one by one, plus edge
cases and error paths that need a device."""
import ctypes

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


def _rows_to_check(M, block_m, n_random=3, seed=0):
    """First/last rows, both sides of the first tile boundary, and a few random rows."""
    rows = {0, M - 1, min(M - 1, block_m - 1), min(M - 1, block_m), M // 2}
    gen = np.random.default_rng(seed)
    rows.update(int(r) for r in gen.integers(0, M, n_random))
    return np.array(sorted(rows), dtype=np.int64)


def _check_rows(g, oracle, A, B, dtype, cfg, alpha, max_a, max_b, rows=None):
    from gpu_util import bf16_to_f64, run_cfg, to_dev
    M, K = A.shape
    N = B.shape[1]
    out = run_cfg(cfg, to_dev(A), to_dev(B), M, N, alpha=alpha)
    rows = _rows_to_check(M, cfg.block_m) if rows is None else rows
    _, ref64 = oracle.gemm_rows(A, B, rows, dtype, alpha=alpha)
    got = bf16_to_f64(out[rows])
    assert np.isfinite(got).all(), "unwritten or non-finite outputs in checked rows"
    err = float(np.max(np.abs(got - ref64)))
    tol = oracle.tolerance(K, max_a, max_b, dtype)
    assert err <= tol, (cfg.describe(), err, tol)
    # every output must have been written (the buffer was poisoned with a NaN pattern)
    assert not np.any((out & 0x7FFF) > 0x7F80), "NaN left in the output"
    return err, tol


def _check_all(g, oracle, A, B, dtype, cfg, alpha, max_a, max_b, Bdev=None):
    """Every element of the product against the oracle (the whole fp64 reference), at the tolerance
    the benchmark states; returns (max error, tolerance)."""
    from gpu_util import bf16_to_f64, run_cfg, to_dev
    M, K = A.shape
    N = B.shape[1]
    out = run_cfg(cfg, to_dev(A), to_dev(B if Bdev is None else Bdev), M, N, alpha=alpha)
    assert not np.any((out & 0x7FFF) > 0x7F80), "NaN left in the output"
    _, ref64 = oracle.gemm(A, B, dtype, alpha=alpha)
    tol = oracle.tolerance(K, max_a, max_b, dtype)
    err = 0.0
    for r0 in range(0, M, 1024):                      # in row blocks: bounded host memory
        err = max(err, float(np.max(np.abs(bf16_to_f64(out[r0:r0 + 1024]) - ref64[r0:r0 + 1024]))))
    assert err <= tol, (cfg.describe(), err, tol)
    return err, tol


@pytest.mark.parametrize("n", [4096, 8192])
def test_config2_square_bf16(g, oracle, n):
    """All n x n outputs of the headline workload, in the launch configuration bench.py times."""
    A, B = wl.config2(n)
    cfg = g.gemm_select(n, n, n, BF16)
    max_a = float(np.abs(wl.bf16_bits_to_f32(A)).max())
    max_b = float(np.abs(wl.bf16_bits_to_f32(B)).max())
    err, tol = _check_all(g, oracle, A, B, BF16, cfg, 1.0, max_a, max_b)
    assert err <= 0.1 * tol          # in practice far inside the bound


@pytest.mark.parametrize("N,K", wl.SKINNY_NK)
def test_config3_skinny_bf16(g, oracle, N, K):
    """Every row for every M."""
    for M in wl.SKINNY_M:
        A, B = wl.config3(M, N, K)
        cfg = g.gemm_select(M, N, K, BF16)
        assert cfg.block_m <= max(128, M), cfg.describe()     # never a 256-row tile for a few tokens
        max_a = float(np.abs(wl.bf16_bits_to_f32(A)).max())
        max_b = float(np.abs(wl.bf16_bits_to_f32(B)).max())
        _check_all(g, oracle, A, B, BF16, cfg, 1.0, max_a, max_b)
        del A, B


def test_config4_fp8_8192(g, oracle):
    """All 8192 x 8192 outputs."""
    n = 8192
    A, B, sa, sb = wl.config4(n)
    alpha = float(sa) * float(sb)
    cfg = g.gemm_select(n, n, n, E4M3)
    # maxima of the real-valued (scale-applied) tensors: 448 * scale by construction
    _check_all(g, oracle, A, B, E4M3, cfg, alpha, 448.0 * float(sa), 448.0 * float(sb))


def test_config5_irregular_shapes(g, oracle):
    shapes = wl.config5_shapes()
    assert len(shapes) == 64 and all(64 <= d <= 16384 and d % 16 == 0 for s in shapes for d in s)
    for i, (M, N, K) in enumerate(shapes):
        A, B = wl.config5(i, shapes)
        cfg = g.gemm_select(M, N, K, BF16)
        rows = _rows_to_check(M, cfg.block_m, n_random=1, seed=i)
        _check_rows(g, oracle, A, B, BF16, cfg, 1.0, 1.0, 1.0, rows=rows)


def test_config5_irregular_shapes_k_contiguous_b(g, oracle):
    """The same 64 shapes with B stored N x K: the K-contiguous selector's picks (other tiles, other
    split and Stream-K choices than above) against sampled oracle rows."""
    from gpu_util import bf16_to_f64, run_cfg, to_dev
    shapes = wl.config5_shapes()
    n_sk = 0
    for i, (M, N, K) in enumerate(shapes):
        A, B = wl.config5(i, shapes)
        cfg = g.gemm_select_ex(M, N, K, BF16, g.GEMM_B_K_CONTIGUOUS)
        n_sk += cfg.stream_k
        rows = _rows_to_check(M, cfg.block_m, n_random=1, seed=100 + i)
        out = run_cfg(cfg, to_dev(A), to_dev(np.ascontiguousarray(B.T)), M, N)
        _, ref64 = oracle.gemm_rows(A, B, rows, BF16)
        err = float(np.max(np.abs(bf16_to_f64(out[rows]) - ref64)))
        assert err <= oracle.tolerance(K, 1.0, 1.0, BF16), (cfg.describe(), err)
        assert not np.any((out & 0x7FFF) > 0x7F80), "NaN left in the output"
    assert n_sk >= 1


def test_fp8_random_every_variant_within_tolerance(g, oracle):
    """Random e4m3 data (not exact in fp32): every variant against the full oracle product."""
    from gpu_util import bf16_to_f64, run_cfg, to_dev
    M, N, K = 272, 528, 1040
    A, B, sa, sb = wl.normal_e4m3(M, N, K, seed=3, case=7)
    alpha = float(sa) * float(sb)
    _, ref64 = oracle.gemm(A, B, E4M3, alpha=alpha)
    tol = oracle.tolerance(K, 448.0 * float(sa), 448.0 * float(sb), E4M3)
    dA, dB = to_dev(A), to_dev(B)
    worst = 0.0
    for idx in range(g.gemm_cfg_count(E4M3)):
        c = g.gemm_cfg_at(idx, M, N, K, E4M3)
        if c is None:
            continue
        out = run_cfg(c, dA, dB, M, N, alpha=alpha)
        err = float(np.max(np.abs(bf16_to_f64(out) - ref64)))
        assert err <= tol, (c.describe(), err, tol)
        worst = max(worst, err)
    assert worst <= 0.05 * tol


@pytest.mark.parametrize("shape", [(1, 8, 8), (1, 16, 8), (3, 8, 16), (17, 24, 40), (1, 4096, 64), (255, 264, 8),
                                   (257, 8, 4104), (33, 1000, 72)])
def test_edge_shapes_bit_exact(g, oracle, shape):
    """Degenerate and ragged shapes, integer data, every legal variant."""
    from gpu_util import run_cfg, to_dev
    M, N, K = shape
    A, B = wl.integer_bf16(M, N, K, seed=5, case=M + N + K, lo=-3, hi=3)
    ref16, _ = oracle.gemm(A, B, BF16, alpha=0.5)
    dA, dB = to_dev(A), to_dev(B)
    n_run = 0
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at(idx, M, N, K, BF16)
        if c is None:
            continue
        out = run_cfg(c, dA, dB, M, N, alpha=0.5)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        n_run += 1
    assert n_run >= 30


def test_padded_leading_dimensions_and_alpha(g, oracle):
    from gpu_util import to_dev, workspace_for
    M, N, K = 200, 264, 328
    lda, ldb, ldc = K + 24, N + 40, N + 8
    A, B = wl.integer_bf16(M, N, K, seed=9)
    Ap = np.full((M, lda), 0x7FC0, np.uint16); Ap[:, :K] = A      # NaN padding must never be read into results
    Bp = np.full((K, ldb), 0x7FC0, np.uint16); Bp[:, :N] = B
    ref16, _ = oracle.gemm(A, B, BF16, alpha=-2.0)
    dA, dB = to_dev(Ap), to_dev(Bp)
    for idx in (0, 5, 60, 130, 170, 200):
        c = g.gemm_cfg_at(idx, M, N, K, BF16)
        if c is None:
            continue
        c.lda, c.ldb, c.ldc, c.alpha = lda, ldb, ldc, -2.0
        workspace_for(c)
        dC = torch.full((M, ldc), 0x1234, dtype=torch.int16, device="cuda")
        g.gemm_run(c, dA, dB, dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16)
        assert np.array_equal(out[:, :N], ref16), c.describe()
        assert np.all(out[:, N:] == 0x1234), "wrote outside the N columns of C"


def test_runs_are_bit_identical_and_split_k_needs_a_workspace(g, oracle):
    from gpu_util import run_cfg, to_dev
    M, N, K = 320, 384, 4096
    A, B = wl.uniform_bf16(M, N, K, seed=12)
    dA, dB = to_dev(A), to_dev(B)
    split = next(c for c in (g.gemm_cfg_at(i, M, N, K, BF16) for i in range(g.gemm_cfg_count(BF16)))
                 if c is not None and c.split_k == 8 and c.block_m == 64)
    a = run_cfg(split, dA, dB, M, N)
    b = run_cfg(split, dA, dB, M, N)
    assert np.array_equal(a, b)                       # slice-ordered reduction: deterministic
    _, ref64 = oracle.gemm(A, B, BF16)
    from gpu_util import bf16_to_f64
    assert np.max(np.abs(bf16_to_f64(a) - ref64)) <= oracle.tolerance(K, 1.0, 1.0, BF16)
    # error path: split-K without a registered (or with a too small) workspace launches nothing
    import gpu_util
    g.gemm_set_workspace(None)
    gpu_util._ws.clear()
    dC = torch.zeros((M, N), dtype=torch.int16, device="cuda")
    rc = g._lib.gemm_run(ctypes.byref(split), ctypes.c_void_p(dA.data_ptr()), ctypes.c_void_p(dB.data_ptr()),
                         ctypes.c_void_p(dC.data_ptr()), None)
    assert rc == -6
    small = torch.empty(16, dtype=torch.float32, device="cuda")
    g.gemm_set_workspace(small)
    rc = g._lib.gemm_run(ctypes.byref(split), ctypes.c_void_p(dA.data_ptr()), ctypes.c_void_p(dB.data_ptr()),
                         ctypes.c_void_p(dC.data_ptr()), None)
    assert rc == -6
    torch.cuda.synchronize()
    assert not dC.any()
    g.gemm_set_workspace(None)


def test_large_shape_16384(g, oracle):
    M, N, K = 16384, 16384, 256
    A, B = wl.uniform_bf16(M, N, K, seed=13)
    cfg = g.gemm_select(M, N, K, BF16)
    _check_rows(g, oracle, A, B, BF16, cfg, 1.0, 1.0, 1.0, rows=np.array([0, 8191, 8192, 16383]))


def test_runs_on_a_side_stream(g, oracle):
    from gpu_util import to_dev
    A, B = wl.config1(integer=True)
    ref16, _ = oracle.gemm(A, B, BF16)
    dA, dB = to_dev(A), to_dev(B)
    cfg = g.gemm_cfg_at(0, 512, 512, 512, BF16)
    s = torch.cuda.Stream()
    dC = torch.zeros((512, 512), dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    g.gemm_run(cfg, dA, dB, dC, stream=s)
    s.synchronize()
    assert np.array_equal(dC.cpu().numpy().view(np.uint16), ref16)


# ---------------- B stored K-contiguous (N x K row-major): the paper's operand layout ----------------

@pytest.mark.parametrize("shape", [(200, 264, 328), (512, 512, 512), (1, 8, 8), (33, 1000, 72)])
def test_k_contiguous_b_every_variant_bit_exact(g, oracle, shape):
    from gpu_util import run_cfg, to_dev
    M, N, K = shape
    A, B = wl.integer_bf16(M, N, K, seed=21, case=M + K)
    ref16, _ = oracle.gemm(A, B, BF16)                   # the oracle always takes B as K x N
    dA, dBt = to_dev(A), to_dev(np.ascontiguousarray(B.T))
    n_run = 0
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at_ex(idx, M, N, K, BF16, g.GEMM_B_K_CONTIGUOUS)
        if c is None:
            continue
        out = run_cfg(c, dA, dBt, M, N)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        n_run += 1
    assert n_run >= 30


def test_k_contiguous_b_fp8_and_padded_ldb(g, oracle):
    from gpu_util import run_cfg, to_dev
    M, N, K = 200, 272, 336
    gen = np.random.default_rng(4)
    vals = np.array([0, 1, 2, 3, 4, -1, -2, -3, -4], dtype=np.float64)
    A = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(M, K))])
    B = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(K, N))])
    ref16, _ = oracle.gemm(A, B, E4M3, alpha=0.25)
    ldb = K + 48
    Bt = np.full((N, ldb), 0x7F, np.uint8)               # NaN codes in the padding
    Bt[:, :K] = B.T
    dA, dBt = to_dev(A), to_dev(Bt)
    for idx in range(g.gemm_cfg_count(E4M3)):
        c = g.gemm_cfg_at_ex(idx, M, N, K, E4M3, g.GEMM_B_K_CONTIGUOUS)
        if c is None:
            continue
        c.ldb = ldb
        out = run_cfg(c, dA, dBt, M, N, alpha=0.25)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))


@pytest.mark.parametrize("M", [1, 16, 100])
def test_weight_streaming_instantiation_and_rotated_k_order(g, oracle, M):
    """A grid of one tile row over weights larger than the memory-side cache runs the weight-streaming instantiation;
    over K-contiguous weights whose row pitch is a power of two of at least 16 KiB (K = 8192 bf16, 16384 fp8; from
    8 KiB, K = 4096 bf16, for the tiles of at most 32 rows) it walks K in an order rotated by tile column (whole
    slabs; also inside every K split).  The test shrinks the cache size in the hardware descriptor so that small
    weights take that path.  Integer operands: any order of the K sum is exact, so every configuration, in both
    layouts, must match the oracle bit for bit.  A second K (the same pitch of the allocation, K itself not a whole
    number of slabs) takes the plain order; at M = 100 the tiles of 64 rows and fewer have several tile rows and run
    the plain instantiation."""
    from gpu_util import run_cfg, to_dev
    hw = g.gemm_hw_get()
    small = g.gemm_hw_get()
    small.mall_bytes = 1 << 20
    N = 1008           # whole 16-byte chunks in both datatypes (a ragged N runs the trimming instantiation instead)
    cases = [(BF16, 8192, 8192), (BF16, 8000, 8192), (BF16, 4096, 4096)]
    if M <= 16:
        cases.append((E4M3, 16384, 16384))
    try:
        g.gemm_hw_set(small)
        for dtype, K, ld in cases:
            if dtype == BF16:
                A, B = wl.integer_bf16(M, N, K, seed=77, case=M + K)
            else:
                gen = np.random.default_rng(M + K)
                vals = np.array([0, 1, 2, 3, 4, -1, -2, -3, -4], dtype=np.float64)
                A = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(M, K))])
                B = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(K, N))])
            ref16, _ = oracle.gemm(A, B, dtype)
            Bt = np.zeros((N, ld), B.dtype)
            Bt[:, :K] = B.T
            for b_layout, dB in ((g.GEMM_B_K_CONTIGUOUS, to_dev(Bt)), (0, to_dev(B))):
                dA = to_dev(A)
                n_one_row = 0
                for idx in range(g.gemm_cfg_count(dtype)):
                    c = g.gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout)
                    if c is None:
                        continue
                    if b_layout:
                        c.ldb = ld
                    out = run_cfg(c, dA, dB, M, N)
                    assert np.array_equal(out, ref16), (c.describe(), K, int((out != ref16).sum()))
                    n_one_row += c.block_m >= M
                assert n_one_row >= 10
    finally:
        g.gemm_hw_set(hw)


def test_k_contiguous_b_square_4096(g, oracle):
    """All 4096 x 4096 outputs with B stored N x K."""
    n = 4096
    A, B = wl.config2(n)
    cfg = g.gemm_select_ex(n, n, n, BF16, g.GEMM_B_K_CONTIGUOUS)
    max_a = float(np.abs(wl.bf16_bits_to_f32(A)).max())
    max_b = float(np.abs(wl.bf16_bits_to_f32(B)).max())
    _check_all(g, oracle, A, B, BF16, cfg, 1.0, max_a, max_b, Bdev=np.ascontiguousarray(B.T))


# ---------------- C = alpha*A*B + beta*C (Section II-A's full definition) ----------------

def test_beta_accumulates_into_c_bit_exact_on_every_path(g, oracle):
    """Integer operands and power-of-two scalars: exact in fp32, so data-parallel, split-K and
    Stream-K epilogues must all reproduce the oracle's alpha*A*B + beta*C_in bit for bit."""
    from gpu_util import to_dev, workspace_for
    M, N, K = 520, 776, 1024
    A, B = wl.integer_bf16(M, N, K, seed=51, case=3)
    gen = np.random.default_rng(52)
    Cin = oracle.encode_bf16(gen.integers(-64, 65, size=(M, N)).astype(np.float64))
    _, prod = oracle.gemm(A, B, BF16, alpha=0.5)
    ref16, _ = oracle.accumulate(prod, -2.0, Cin)
    dA, dB = to_dev(A), to_dev(B)
    seen = set()
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at(idx, M, N, K, BF16)
        if c is None:
            continue
        path = "streamk" if c.stream_k else ("splitk" if c.split_k > 1 else "dp")
        if c.split_k > 4:
            continue
        c.alpha, c.beta = 0.5, -2.0
        workspace_for(c)
        dC = to_dev(Cin).clone()
        g.gemm_run(c, dA, dB, dC)
        torch.cuda.synchronize()
        out = dC.cpu().numpy().view(np.uint16)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        seen.add(path)
    assert seen == {"dp", "splitk", "streamk"}


def test_beta_random_data_padded_ldc_within_tolerance(g, oracle):
    from gpu_util import bf16_to_f64, to_dev, workspace_for
    M, N, K = 1000, 1512, 2048
    A, B = wl.config2(2048)
    A, B = np.ascontiguousarray(A[:M, :K]), np.ascontiguousarray(B[:K, :N])
    gen = np.random.default_rng(53)
    Cin = wl.f32_to_bf16_bits(gen.standard_normal((M, N), dtype=np.float32) * 30.0)
    alpha, beta = 0.75, 1.25
    _, prod = oracle.gemm(A, B, BF16, alpha=alpha)
    _, ref64 = oracle.accumulate(prod, beta, Cin)
    # the benchmark spec's bound on the product, plus the rounding of the beta*C term in fp32 and bf16
    tol = oracle.tolerance(K, float(np.abs(bf16_to_f64(A)).max()), float(np.abs(bf16_to_f64(B)).max()), BF16)
    ldc = N + 24
    Cp = np.full((M, ldc), 0x1234, np.uint16)
    Cp[:, :N] = Cin
    c = g.gemm_select(M, N, K, BF16)
    c.ldc, c.alpha, c.beta = ldc, alpha, beta
    workspace_for(c)
    dC = to_dev(Cp)
    g.gemm_run(c, to_dev(A), to_dev(B), dC)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().view(np.uint16)
    assert np.abs(bf16_to_f64(out[:, :N]) - ref64).max() <= tol
    assert np.all(out[:, N:] == 0x1234)


# ---------------- gemm_run under HIP graph capture ----------------

def test_graph_replays_match_eager_on_every_path(g, oracle):
    """gemm_run only enqueues kernels (no allocation, no memset), so it can be captured.  Each
    replay runs on fresh inputs written between replays by ordinary eager work and is compared
    with the oracle: data-parallel, split-K (two kernels) and Stream-K (two kernels)."""
    from gpu_util import to_dev, workspace_for
    M, N, K = 520, 776, 1024
    picks = {}
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at(idx, M, N, K, BF16)
        if c is None:
            continue
        path = "streamk" if c.stream_k else ("splitk" if c.split_k == 4 else "dp" if c.split_k == 1 else None)
        if path and path not in picks and (c.block_m, c.block_n) == (128, 128):
            picks[path] = c
    assert set(picks) == {"dp", "splitk", "streamk"}
    cases = []
    for r in range(3):
        A, B = wl.integer_bf16(M, N, K, seed=81, case=r)
        cases.append((A, B, oracle.gemm(A, B, BF16)[0]))
    dA, dB = to_dev(cases[0][0]).clone(), to_dev(cases[0][1]).clone()
    dC = torch.empty((M, N), dtype=torch.int16, device="cuda")
    for path, c in picks.items():
        workspace_for(c)
        g.gemm_run(c, dA, dB, dC)                       # warm-up outside capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            g.gemm_run(c, dA, dB, dC)
        for A, B, ref16 in cases:
            dA.copy_(to_dev(A))
            dB.copy_(to_dev(B))
            dC.fill_(0x7FC0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            out = dC.cpu().numpy().view(np.uint16)
            assert np.array_equal(out, ref16), (path, c.describe())
        del graph


def test_very_deep_reduction_bit_exact(g, oracle):
    """K = 131072 with a 64 x 64 output: 2048 slabs per tile, split-K up to 32 and Stream-K; integer
    operands keep every fp32 partial sum exact (|sum| <= 16 K < 2^24)."""
    from gpu_util import run_cfg, to_dev
    M, N, K = 64, 64, 131072
    A, B = wl.integer_bf16(M, N, K, seed=91)
    ref16, _ = oracle.gemm(A, B, BF16)
    dA, dB = to_dev(A), to_dev(B)
    kinds = set()
    cfgs = [g.gemm_select(M, N, K, BF16)]
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at(idx, M, N, K, BF16)
        if c is not None and (c.block_m, c.block_n) in ((64, 64), (16, 16), (32, 32)) and (c.split_k in (1, 32) or c.stream_k):
            cfgs.append(c)
    for c in cfgs:
        out = run_cfg(c, dA, dB, M, N)
        assert np.array_equal(out, ref16), (c.describe(), int((out != ref16).sum()))
        kinds.add("streamk" if c.stream_k else "split%d" % c.split_k)
    assert {"split1", "split32", "streamk"} <= kinds
