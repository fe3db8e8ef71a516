"""Host side of the grouped launch: the selection model against the model oracle, the plan's
table (tile ranges, empty groups, per-group rasterisation) and the group search, argument
errors.  No GPU."""
import ctypes

import pytest

from oracle import selector_model as sm
from paper_2512_04226_amd import binding as g
from paper_2512_04226_amd import workloads as wl
from test_selector_model import _hw_dict, _variant_dict

SETS = [
    [(300, 1024, 512), (0, 1024, 512), (40, 512, 1024), (1000, 2048, 256)],
    [(m, 4096, 2048) for m in wl.routed_rows(8, 4096, seed=11)],
    [(m, 1024, 7168) for m in wl.routed_rows(32, 2048, seed=12, skew=0.3)],
    [(16, 28672, 8192)],
    [(4096, 4096, 4096), (8, 64, 64)],
]


@pytest.mark.parametrize("b_layout", [0, 1])
@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_grouped_prediction_and_pick_match_the_oracle(dtype, b_layout):
    hw = _hw_dict(g)
    for shapes in SETS:
        if dtype == 1:
            shapes = [(m, n, k) for (m, n, k) in shapes if n % 16 == 0 and k % 16 == 0]
        probs = g.make_problems(shapes, b_layout)
        best, n_legal = None, 0
        for vid in range(g.gemm_variant_count(dtype)):
            c = g.gemm_cfg_at_grouped(vid, probs, dtype, b_layout)
            if c is None:
                continue
            n_legal += 1
            assert c.groups == len(shapes) and c.split_k == 1 and not c.stream_k and c.batch == 1
            assert c.kernel_id == vid and c.b_layout == b_layout
            live = [s for s in shapes if s[0] > 0]
            assert (c.M, c.N, c.K) == tuple(max(s[i] for s in live) for i in range(3))
            l_total, group_m = sm.predict_grouped(hw, dtype, shapes, _variant_dict(c), b_layout)
            assert c.predicted_us == pytest.approx(l_total / (hw["clk_ghz"] * 1e3), rel=1e-9)
            table, total = g.gemm_grouped_plan(c, probs_with_fake_pointers(shapes, b_layout))
            assert [r.group_m for r in table] == [group_m[i] for i in plan_order(shapes)]
            if best is None or l_total < best[0] * (1 - 1e-12):
                best = (l_total, vid)
        assert n_legal > 10
        pick = g.gemm_select_grouped(probs, dtype, b_layout)
        assert pick.kernel_id == best[1], (shapes, pick.describe())


def plan_order(shapes):
    """The table's record order: descending K, ties in the caller's order."""
    return sorted(range(len(shapes)), key=lambda i: -shapes[i][2])


def probs_with_fake_pointers(shapes, b_layout=0):
    """Problems with well-aligned non-NULL addresses that are never dereferenced on the host."""
    probs = g.make_problems(shapes, b_layout)
    for i, p in enumerate(probs):
        p.A, p.B, p.C = 0x10000 * (3 * i + 1), 0x10000 * (3 * i + 2), 0x10000 * (3 * i + 3)
    return probs


def test_a_single_group_reduces_to_waves_times_the_full_tile_latency():
    """One group: Algorithm 9 as printed -- waves times the tile latency, plus the launch."""
    hw = _hw_dict(g)
    M, N, K = 8192, 8192, 8192
    c = g.gemm_cfg_at_grouped(0, g.make_problems([(M, N, K)]), 0)
    p = g.gemm_predict(g.gemm_cfg_at(0, M, N, K, 0))       # variant 0, split 1, the same shape
    assert p.waves == 4
    assert c.predicted_us * hw["clk_ghz"] * 1e3 == pytest.approx(hw["launch_clk"] + 4 * p.l_tile, rel=1e-9)


@pytest.mark.parametrize("xcd_remap", [1, 0])
def test_plan_table_slots_and_workgroup_to_tile_mapping(xcd_remap):
    """Every tile of every group is computed by exactly one workgroup; each group takes the same
    slot range on every XCD and XCD x (= workgroup id mod X) owns a contiguous chunk of it."""
    shapes = [(0, 512, 256), (300, 1024, 512), (0, 1024, 512), (40, 512, 1024), (1000, 2048, 256), (0, 64, 64)]
    probs = probs_with_fake_pointers(shapes)
    c = g.gemm_select_grouped(probs, 0)
    c.xcd_remap = xcd_remap
    X = g.gemm_hw_get().n_xcd if xcd_remap else 1
    table, grid = g.gemm_grouped_plan(c, probs)
    bm, bn = c.block_m, c.block_n
    start = 0
    assert plan_order(shapes) == [3, 1, 2, 0, 4, 5]
    for r, i in zip(table, plan_order(shapes)):
        M, N, K = shapes[i]
        assert (r.A, r.B, r.C) == (probs[i].A, probs[i].B, probs[i].C)
        assert (r.M, r.N, r.K, r.lda, r.ldb, r.ldc) == (M, N, K, K, N, N)
        assert r.tiles_m == -(-M // bm) and r.tiles_n == -(-N // bn) and r.tile_start == start
        start += -(-(r.tiles_m * r.tiles_n) // X)
    assert grid == start * X and table[0].tile_start == 0 and table[-1].M == 0 and table[-1].tile_start == start
    seen, idle, last = {}, 0, {}
    for wg in range(grid):
        rec, tm, tn = g.gemm_grouped_locate(c, table, wg)
        if rec < 0:
            idle += 1
            continue
        r = table[rec]
        assert r.M > 0 and 0 <= tm < r.tiles_m and 0 <= tn < r.tiles_n
        assert (rec, tm, tn) not in seen
        seen[(rec, tm, tn)] = wg % X
        # an XCD meets the records in table order (longest K first)
        assert last.get(wg % X, 0) <= rec
        last[wg % X] = rec
    assert len(seen) == sum(r.tiles_m * r.tiles_n for r in table)
    assert idle == grid - len(seen) and idle <= (X - 1) * sum(1 for r in table if r.M > 0)
    if X > 1:
        # a group with at least X tiles is spread over every XCD
        for rec, r in enumerate(table):
            if r.tiles_m * r.tiles_n >= X:
                assert {x for (rr, _, _), x in seen.items() if rr == rec} == set(range(X))
    with pytest.raises(g.GemmError):
        g.gemm_grouped_locate(c, table, grid)
    # the records are plain bytes: the device copy is these 64-byte records
    assert len(bytes(table)) == 64 * len(shapes)


def test_grouped_argument_errors():
    shapes = [(300, 1024, 512), (40, 512, 1024)]
    probs = probs_with_fake_pointers(shapes)
    cfg = g.gemm_cfg()
    f = g._lib.gemm_select_grouped
    assert f(2, probs, 0, 0, None) == -1
    assert f(2, None, 0, 0, ctypes.byref(cfg)) == -1
    assert f(0, probs, 0, 0, ctypes.byref(cfg)) == -2
    assert f(5000, probs, 0, 0, ctypes.byref(cfg)) == -2
    assert f(2, probs, 9, 0, ctypes.byref(cfg)) == -3
    assert f(2, probs, 0, 3, ctypes.byref(cfg)) == -4
    ragged = probs_with_fake_pointers([(300, 1020, 512), (40, 512, 1023)])
    assert f(2, ragged, 0, 0, ctypes.byref(cfg)) == 0           # N and K need not be whole 16-byte chunks
    neg = probs_with_fake_pointers([(-1, 1024, 512), (40, 512, 1024)])
    assert f(2, neg, 0, 0, ctypes.byref(cfg)) == -2
    empty = probs_with_fake_pointers([(0, 1024, 512), (0, 512, 1024)])
    assert f(2, empty, 0, 0, ctypes.byref(cfg)) == -2           # nothing to select for
    assert g._lib.gemm_cfg_at_grouped(-1, 2, probs, 0, 0, ctypes.byref(cfg)) == -9
    assert g._lib.gemm_cfg_at_grouped(10 ** 6, 2, probs, 0, 0, ctypes.byref(cfg)) == -9

    c = g.gemm_select_grouped(probs, 0)
    table, total = g.gemm_grouped_plan(c, probs)
    plan = g._lib.gemm_grouped_plan
    out = (g.gemm_group_rec * 2)()
    tot = ctypes.c_int64()
    assert plan(ctypes.byref(c), 2, probs, None, ctypes.byref(tot)) == -1
    assert plan(ctypes.byref(c), 3, probs, out, ctypes.byref(tot)) == -4        # cfg is for 2 groups
    plain = g.gemm_select(300, 1024, 512, 0)
    assert plan(ctypes.byref(plain), 2, probs, out, ctypes.byref(tot)) == -4    # not a grouped cfg
    old = c.copy()
    old.abi_version = 3
    assert plan(ctypes.byref(old), 2, probs, out, ctypes.byref(tot)) == -7
    unaligned = probs_with_fake_pointers(shapes)
    unaligned[1].B = 0x10008
    assert plan(ctypes.byref(c), 2, unaligned, out, ctypes.byref(tot)) == -5
    null = probs_with_fake_pointers(shapes)
    null[0].C = None
    assert plan(ctypes.byref(c), 2, null, out, ctypes.byref(tot)) == -1
    short = probs_with_fake_pointers(shapes)
    short[0].lda = 504
    assert plan(ctypes.byref(c), 2, short, out, ctypes.byref(tot)) == -2
    split = c.copy()
    split.split_k = 2
    assert plan(ctypes.byref(split), 2, probs, out, ctypes.byref(tot)) == -4
    # an empty group may carry NULL pointers
    with_empty = probs_with_fake_pointers([(300, 1024, 512), (0, 512, 1024)])
    with_empty[1].A = with_empty[1].B = with_empty[1].C = None
    c2 = g.gemm_select_grouped(with_empty, 0)
    t2, _ = g.gemm_grouped_plan(c2, with_empty)
    empty_rec = [r for r in t2 if r.M == 0][0]
    assert empty_rec.tiles_m == 0 and empty_rec.A == 0

    # gemm_run_grouped validates the host table again and launches nothing on error (no GPU here:
    # every call below must return before any HIP call)
    run = g._lib.gemm_run_grouped
    dev = ctypes.c_void_p(0x100000)
    assert run(ctypes.byref(c), 2, table, None, None) == -1
    assert run(ctypes.byref(c), 2, table, ctypes.c_void_p(0x100008), None) == -5
    tampered = (g.gemm_group_rec * 2)()
    ctypes.memmove(tampered, table, 128)
    tampered[1].tile_start += 1
    assert run(ctypes.byref(c), 2, tampered, dev, None) == -4
    ctypes.memmove(tampered, table, 128)
    tampered[0].tiles_n += 1
    assert run(ctypes.byref(c), 2, tampered, dev, None) == -4
    ctypes.memmove(tampered, table, 128)
    tampered[0].ldc = 8
    assert run(ctypes.byref(c), 2, tampered, dev, None) == -2
    # gemm_run refuses a grouped cfg
    assert g._lib.gemm_run(ctypes.byref(c), dev, dev, dev, None) == -4
