"""GPU parity of the Stream-K path (workers' partial tiles + summation pass) against the CPU oracle."""
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


def _base_cfgs(g, M, N, K, dtype, b_layout=0):
    """One split_k = 1, non-stream-K cfg per variant."""
    out = []
    for idx in range(g.gemm_cfg_count(dtype)):
        c = g.gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout)
        if c is not None and c.split_k == 1 and not c.stream_k:
            out.append(c)
    return out


def _with_workers(g, c, G):
    """cfg c turned into a stream-K cfg with G workers, or None when that is not a legal plan."""
    s = c.copy()
    s.stream_k, s.sk_workers = 1, G
    try:
        g.gemm_stream_k_plan(s)
    except g.GemmError:
        return None
    return s


WORKER_COUNTS = (3, 5, 7, 12, 20, 33, 100, 255, 700)


@pytest.mark.parametrize("shape", [(520, 776, 1024), (200, 264, 2064), (1040, 520, 328)])
@pytest.mark.parametrize("b_layout", [0, 1])
def test_bf16_every_variant_hand_set_workers_bit_exact(g, oracle, shape, b_layout):
    """Integer operands: the fp32 sums are exact whatever the split, so every worker count must
    reproduce the oracle bit for bit.  Ragged M, N and a K that is not a multiple of the slab."""
    from gpu_util import run_cfg, to_dev
    M, N, K = shape
    A, B = wl.integer_bf16(M, N, K, seed=31, case=M + K)
    ref16, _ = oracle.gemm(A, B, BF16)
    dA = to_dev(A)
    dB = to_dev(np.ascontiguousarray(B.T) if b_layout else B)
    n_run, two_seg, whole = 0, 0, 0
    for c in _base_cfgs(g, M, N, K, BF16, b_layout):
        done = 0
        for G in WORKER_COUNTS:
            s = _with_workers(g, c, G)
            if s is None:
                continue
            for w in range(G):
                segs = g.gemm_stream_k_segments(s, w)
                two_seg += len(segs) == 2
                whole += any(x.complete for x in segs)
            print("stream-K", shape, b_layout, s.describe(), flush=True)
            out = run_cfg(s, dA, dB, M, N)
            assert np.array_equal(out, ref16), (s.describe(), int((out != ref16).sum()))
            n_run += 1
            done += 1
            if done == 3:
                break
    assert n_run >= 60 and two_seg > 0


def test_fp8_every_variant_hand_set_workers_bit_exact(g, oracle):
    from gpu_util import run_cfg, to_dev
    M, N, K = 520, 784, 2064
    gen = np.random.default_rng(5)
    vals = np.array([0, 1, 2, 3, 4, -1, -2, -3, -4], dtype=np.float64)
    A = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(M, K))])
    B = oracle.encode_e4m3(vals[gen.integers(0, 9, size=(K, N))])
    ref16, _ = oracle.gemm(A, B, E4M3, alpha=0.5)
    for b_layout in (0, 1):
        dA, dB = to_dev(A), to_dev(np.ascontiguousarray(B.T) if b_layout else B)
        n_run = 0
        for c in _base_cfgs(g, M, N, K, E4M3, b_layout):
            done = 0
            for G in WORKER_COUNTS:
                s = _with_workers(g, c, G)
                if s is None:
                    continue
                print("stream-K fp8", b_layout, s.describe(), flush=True)
                out = run_cfg(s, dA, dB, M, N, alpha=0.5)
                assert np.array_equal(out, ref16), (s.describe(), int((out != ref16).sum()))
                n_run += 1
                done += 1
                if done == 2:
                    break
        assert n_run >= 25


def test_enumerated_stream_k_cfgs_random_data_within_tolerance(g, oracle):
    """The device's own worker counts on a problem with a partial last wave (17 x 17 tiles of
    256 x 256 on 256 CUs), N(0,1) data, sampled rows against the oracle; repeated runs identical."""
    from gpu_util import bf16_to_f64, run_cfg, to_dev
    M = N = 4352
    K = 2048
    gen = np.random.default_rng([41, 0])
    A = wl.f32_to_bf16_bits(gen.standard_normal((M, K), dtype=np.float32))
    B = wl.f32_to_bf16_bits(gen.standard_normal((K, N), dtype=np.float32))
    rows = np.unique(np.concatenate([np.arange(0, M, 97), [255, 256, 4095, 4096, 4351]]))
    ref16, ref64 = oracle.gemm_rows(A, B, rows, BF16)
    tol = oracle.tolerance(K, float(np.abs(bf16_to_f64(A)).max()), float(np.abs(bf16_to_f64(B)).max()), BF16)
    dA, dB = to_dev(A), to_dev(B)
    n_run = 0
    for idx in range(g.gemm_cfg_count(BF16)):
        c = g.gemm_cfg_at(idx, M, N, K, BF16)
        if c is None or not c.stream_k:
            continue
        print("stream-K enumerated", c.describe(), flush=True)
        out = run_cfg(c, dA, dB, M, N)
        err = np.abs(bf16_to_f64(out[rows]) - ref64).max()
        assert err <= tol, (c.describe(), err, tol)
        if n_run % 8 == 0:
            again = run_cfg(c, dA, dB, M, N)
            assert np.array_equal(out, again), c.describe()
        n_run += 1
    assert n_run >= 10


def test_stream_k_padded_leading_dimensions_alpha_and_workspace_errors(g, oracle):
    from gpu_util import to_dev, workspace_for
    M, N, K = 300, 520, 1096
    A, B = wl.integer_bf16(M, N, K, seed=33, case=7)
    ref16, _ = oracle.gemm(A, B, BF16, alpha=0.25)
    lda, ldb, ldc = K + 24, N + 40, N + 16
    Ap = np.full((M, lda), 0x7FC0, np.uint16); Ap[:, :K] = A
    Bp = np.full((K, ldb), 0x7FC0, np.uint16); Bp[:, :N] = B
    dA, dB = to_dev(Ap), to_dev(Bp)
    c = next(x for x in _base_cfgs(g, M, N, K, BF16) if (x.block_m, x.block_n) == (128, 128))
    s = _with_workers(g, c, 5)          # 3 x 5 = 15 tiles: 0 left over -> not a plan
    assert s is None
    s = _with_workers(g, c, 4)          # 3 tiles left over, cut into 4 ranges
    assert s is not None
    s.lda, s.ldb, s.ldc, s.alpha = lda, ldb, ldc, 0.25
    g.gemm_set_workspace(None)
    dC = torch.full((M, ldc), 0x1234, dtype=torch.int16, device="cuda")
    with pytest.raises(g.GemmError):
        g.gemm_run(s, dA, dB, dC)
    small = torch.empty(16, dtype=torch.float32, device="cuda")
    g.gemm_set_workspace(small)
    with pytest.raises(g.GemmError):
        g.gemm_run(s, dA, dB, dC)
    from gpu_util import _ws
    _ws.clear()
    workspace_for(s)
    g.gemm_run(s, dA, dB, dC)
    torch.cuda.synchronize()
    out = dC.cpu().numpy().view(np.uint16)
    assert np.array_equal(out[:, :N], ref16)
    assert np.all(out[:, N:] == 0x1234)      # the padding of C is untouched
