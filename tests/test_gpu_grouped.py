"""GPU parity of grouped launches (several products of different shapes in one grid) against
the CPU oracle, one plain product per group."""
import numpy as np
import pytest
import torch

from paper_2512_04226_amd import workloads as wl

pytestmark = pytest.mark.gpu

BF16, E4M3, FP16 = 0, 1, 2
POISON = 0x7FC0


@pytest.fixture(scope="module")
def g():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04226_amd import binding
    return binding


def _operands(shapes, dtype, seed, b_layout=0, integer=True):
    """Per group (A bits, B bits as the oracle wants them (K x N), B bits as stored)."""
    out = []
    for i, (M, N, K) in enumerate(shapes):
        if dtype == E4M3:
            A, B, sa, sb = wl.normal_e4m3(max(M, 1), N, K, seed=seed, case=i)
        elif integer:
            A, B = (wl.integer_fp16 if dtype == FP16 else wl.integer_bf16)(max(M, 1), N, K, seed=seed, case=i)
        else:
            A, B = (wl.normal_fp16 if dtype == FP16 else wl.normal_bf16)(max(M, 1), N, K, seed=seed, case=i)
        A = A[:M]
        out.append((A, B, np.ascontiguousarray(B.T) if b_layout else B))
    return out


def _run(g, cfg, shapes, ops, beta_in=None, pad=0):
    """All groups' C live in one poisoned buffer with guard gaps between them; returns the
    per-group outputs and checks that nothing outside them was written."""
    from gpu_util import to_dev
    dev = [(to_dev(A) if A.shape[0] else None, to_dev(Bs), None) for (A, _, Bs) in ops]
    gap = 64
    sizes = [M * (N + pad) for (M, N, K) in shapes]
    offs, pos = [], gap
    for s in sizes:
        offs.append(pos)
        pos += (s + gap + 7) // 8 * 8
    buf = torch.full((pos,), POISON, dtype=torch.int16, device="cuda")
    if beta_in is not None:
        for o, (M, N, K), cin in zip(offs, shapes, beta_in):
            if M:
                buf[o:o + M * (N + pad)].view(M, N + pad)[:, :N] = torch.from_numpy(cin.view(np.int16)).cuda()
    tensors = []
    for (A, B, _), o, (M, N, K) in zip(dev, offs, shapes):
        tensors.append((A, B, buf[o:] if M else None))
    probs = g.make_problems(shapes, cfg.b_layout, tensors)
    for p, (M, N, K) in zip(probs, shapes):
        p.ldc = N + pad
    table, total = g.gemm_grouped_plan(cfg, probs)
    dtab = g.table_to_device(table)
    g.gemm_run_grouped(cfg, table, dtab)
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    outs, mask = [], np.ones(pos, dtype=bool)
    for o, (M, N, K) in zip(offs, shapes):
        blk = host[o:o + M * (N + pad)].reshape(M, N + pad)
        outs.append(blk[:, :N].copy())
        m2 = mask[o:o + M * (N + pad)].reshape(M, N + pad)
        m2[:, :N] = False
    assert np.all(host[mask] == POISON), "a grouped launch wrote outside its groups' outputs"
    return outs


RAGGED = [(300, 1032, 520), (0, 1024, 512), (40, 520, 1096), (1000, 264, 256), (1, 8, 8), (77, 2048, 72)]


@pytest.mark.parametrize("b_layout", [0, 1])
def test_grouped_every_variant_bit_exact_on_ragged_groups(g, oracle, b_layout):
    ops = _operands(RAGGED, BF16, seed=81, b_layout=b_layout)
    refs = oracle.gemm_grouped([(A, B) for (A, B, _) in ops], BF16)
    probs = g.make_problems(RAGGED, b_layout)
    n_run = 0
    for vid in range(g.gemm_variant_count(BF16)):
        c = g.gemm_cfg_at_grouped(vid, probs, BF16, b_layout)
        if c is None:
            continue
        outs = _run(g, c, RAGGED, ops)
        for i, (out, (ref16, _)) in enumerate(zip(outs, refs)):
            assert np.array_equal(out, ref16), (c.describe(), i, RAGGED[i], int((out != ref16).sum()))
        n_run += 1
    assert n_run >= 40


def test_grouped_routed_rows_many_groups_selected_cfg_and_tolerance(g, oracle):
    """64 groups with routing-like row counts (some empty), shared N and K; the analytic pick;
    random operands within the product tolerance; padded ldc."""
    rows = wl.routed_rows(64, 3000, seed=5, skew=0.5)
    assert len(rows) == 64 and sum(rows) == 3000 and len(set(rows)) > 8
    shapes = [(m, 512, 1024) for m in rows]
    ops = _operands(shapes, BF16, seed=82, integer=False)
    pick = g.gemm_select_grouped(g.make_problems(shapes), BF16)
    outs = _run(g, pick, shapes, ops, pad=24)
    for (A, B, _), out, (M, N, K) in zip(ops, outs, shapes):
        if M == 0:
            continue
        _, ref64 = oracle.gemm(A, B, BF16)
        got = (out.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        tol = oracle.tolerance(K, float(np.abs(oracle.decode(A, BF16)).max()), float(np.abs(oracle.decode(B, BF16)).max()), BF16)
        assert np.max(np.abs(got - ref64)) <= tol


def test_grouped_fp8_fp16_and_beta(g, oracle):
    shapes = [(200, 1024, 512), (0, 256, 256), (72, 272, 1040), (513, 528, 128)]
    # fp8: every operand is quantised to the full e4m3 range (max |code value| = 448); a grouped
    # launch has one alpha, here the scale that maps both ranges back to [-1, 1]
    ops = _operands(shapes, E4M3, seed=83)
    pick = g.gemm_select_grouped(g.make_problems(shapes), E4M3)
    pick.alpha = 1.0 / (448.0 * 448.0)
    outs = _run(g, pick, shapes, ops)
    for (A, B, _), out, (M, N, K) in zip(ops, outs, shapes):
        if M == 0:
            continue
        _, ref64 = oracle.gemm(A, B, E4M3, alpha=float(np.float32(pick.alpha)))
        got = (out.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        assert np.max(np.abs(got - ref64)) <= oracle.tolerance(K, 1.0, 1.0, E4M3)
    # fp16, K-contiguous B, beta = -0.5 on integer data: exactly one correct result
    ops = _operands(shapes, FP16, seed=84, b_layout=1)
    pick = g.gemm_select_grouped(g.make_problems(shapes, 1), FP16, 1)
    pick.alpha, pick.beta = 0.25, -0.5
    cins = [wl.f32_to_fp16_bits(np.random.default_rng([85, i]).integers(-8, 9, size=(M, N)).astype(np.float32))
            for i, (M, N, K) in enumerate(shapes)]
    outs = _run(g, pick, shapes, ops, beta_in=cins)
    for (A, B, _), out, cin, (M, N, K) in zip(ops, outs, cins, shapes):
        if M == 0:
            continue
        _, ref64 = oracle.gemm(A, B, FP16, alpha=0.25)
        want, _ = oracle.accumulate(ref64, -0.5, cin, FP16)
        assert np.array_equal(out, want)


def test_grouped_launch_of_empty_groups_only_is_a_no_op(g):
    shapes = [(300, 1024, 512), (0, 512, 1024)]
    c = g.gemm_select_grouped(g.make_problems(shapes), BF16)
    # the same cfg with every group empty: the plan has no tile and the run returns without a launch
    empty = g.make_problems([(0, 1024, 512), (0, 512, 1024)])
    table, total = g.gemm_grouped_plan(c, empty)
    assert total == 0
    g.gemm_run_grouped(c, table, g.table_to_device(table))
    torch.cuda.synchronize()
