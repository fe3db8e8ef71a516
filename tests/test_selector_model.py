"""Pins for the printed algorithms in the model checker (oracle/selector_model.py): the values the paper
prints and the closed forms its algorithms imply; then the library's model terms against the checker's
composition over many shapes and every configuration (a breadth check -- the composed readings themselves are
pinned to hand-worked numbers, for the checker and for the library separately, in test_model_goldens.py)."""
import math
import os

import pytest

from oracle import selector_model as sm

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_examples.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        line = line.split(";")[0].strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split("=")
        out[k.strip()] = v.strip()
    return out


def test_worked_tiling_example_section_2a():
    g = _gold()
    M, N, n_cu = int(g["example_M"]), int(g["example_N"]), int(g["example_n_cu"])
    tm, tn, tk = (int(x) for x in g["small_tile"].split())
    active, omega, t_out = sm.alg4_occupancy(M, N, tm, tn, n_cu)
    assert t_out == int(g["small_tile_output_tiles"]) and omega == 1
    assert active == 0          # the printed modulo gives 0 exactly where the text says "one tile per CU"
    assert tm * tn * tk == int(g["small_tile_volume"])
    tm, tn, tk = (int(x) for x in g["large_tile"].split())
    active, omega, t_out = sm.alg4_occupancy(M, N, tm, tn, n_cu)
    assert t_out == int(g["large_tile_output_tiles"]) and omega == 1 and active == 1
    assert tm * tn * tk == int(g["large_tile_volume"])


def test_factorisation_example_section_4c():
    g = _gold()
    want = [tuple(int(x) for x in p.split("x")) for p in g["factor_example_pairs"].split()]
    assert sm.alg6_factorizations(int(g["factor_example_cus"])) == want
    for n in (1, 7, 32, 38, 256, 304):
        F = sm.alg6_factorizations(n)
        assert all(a * b == n for a, b in F) and len(set(F)) == len(F)
        assert len(F) == sum(1 for i in range(1, n + 1) if n % i == 0)


def test_alg3_counts():
    # 256x256x64 tile of 32x32x16 instructions: 8*8*4; ceilings on ragged tiles
    assert sm.alg3_compute_latency(32, 32, 16, 256, 256, 64, 32.0) == (256, 8192.0)
    assert sm.alg3_compute_latency(32, 32, 8, 48, 16, 20, 1.0)[0] == 2 * 1 * 3
    n, l = sm.alg3_compute_latency(16, 16, 32, 16, 64, 128, 16.0)
    assert n == 16 and l == 256.0


def test_alg4_waves_and_tail():
    assert sm.alg4_occupancy(4096, 4096, 256, 256, 256) == (0, 1, 256)
    assert sm.alg4_occupancy(8192, 8192, 256, 256, 256) == (0, 4, 1024)
    assert sm.alg4_occupancy(4096, 4096 + 1, 256, 256, 256) == (16, 2, 272)
    assert sm.alg4_occupancy(1, 28672, 16, 256, 256) == (112, 1, 112)
    assert sm.alg4_occupancy(300, 300, 128, 128, 304) == (9, 1, 9)


def test_alg5_closed_forms():
    # square s x s cache tile of square workgroup tiles: h = 1 - 1/s; 1 x 1 gives 0
    for s in (1, 2, 4, 16):
        assert sm.alg5_hit_rate(s, s, 128, 128, 64) == pytest.approx(1 - 1 / s)
    assert sm.alg5_hit_rate(1, 1, 256, 64, 32) == 0
    # K_T cancels; a 4 x 8 tile of 256 x 256: U = 12, R = 64
    assert sm.alg5_hit_rate(4, 8, 256, 256, 64) == pytest.approx(1 - 12 / 64)
    assert sm.alg5_hit_rate(4, 8, 256, 256, 64) == sm.alg5_hit_rate(4, 8, 256, 256, 16)
    # asymmetric tiles: transposing the cache tile with the workgroup tile leaves h unchanged
    assert sm.alg5_hit_rate(2, 8, 64, 256, 32) == pytest.approx(sm.alg5_hit_rate(8, 2, 256, 64, 32))
    for fm, fn in sm.alg6_factorizations(32):
        assert 0 <= sm.alg5_hit_rate(fm, fn, 128, 64, 64) <= 1


def test_alg7_structure():
    base = dict(ld_cu=1000.0, C=64, H1=0.5, H2=0.5, R_L1=10.0, R_1=400.0, R_2=300.0, R_MEM=100.0, L_lat=50.0)
    v = sm.alg7_memory_latency(**base)
    terms = [1000 / 10.0, 64000 / 400.0, 32000 / 300.0, 16000 / 100.0 + 50.0]
    assert v == pytest.approx(max(terms)) and v == pytest.approx(210.0)
    assert v >= base["ld_cu"] / base["R_L1"]
    # non-increasing in either hit rate
    for k in ("H1", "H2"):
        prev = None
        for h in (0.0, 0.3, 0.6, 0.9, 1.0):
            cur = sm.alg7_memory_latency(**dict(base, **{k: h}))
            assert prev is None or cur <= prev + 1e-12
            prev = cur
    # with perfect Mem1 hits only issue, Mem1 bandwidth and the bare latency remain
    assert sm.alg7_memory_latency(**dict(base, H1=1.0)) == pytest.approx(max(100.0, 160.0, 50.0))


def test_alg8_alg9_structure():
    # K <= k_t: no loop iterations, only prologue + epilogue
    assert sm.alg8_tile_latency(64, 64, 10.0, 99.0, 4, 16, 16, 8.0) == pytest.approx(10.0 + 4 * 256 / 8.0)
    # one more K slab adds exactly max(l_compute, l_mem)
    a = sm.alg8_tile_latency(640, 64, 10.0, 30.0, 1, 16, 16, 8.0)
    b = sm.alg8_tile_latency(704, 64, 10.0, 30.0, 1, 16, 16, 8.0)
    assert b - a == pytest.approx(30.0)
    assert sm.alg9_total_latency(8192, 8192, 256, 256, 256, 7.0) == pytest.approx(4 * 7.0)
    assert sm.alg9_total_latency(256, 256, 16, 16, 256, 7.0) == pytest.approx(7.0)
    assert sm.alg9_total_latency(256, 272, 16, 16, 256, 7.0) == pytest.approx(2 * 7.0)


# ---------------- the shipped selector's terms against the oracle's composition ----------------

def _hw_dict(g):
    hw = g.gemm_hw_get()
    d = {name: getattr(hw, name) for name, _ in hw._fields_ if name not in ("l_mi_clk", "reserved0")}
    d["l_mi_clk"] = [[hw.l_mi_clk[i][j] for j in range(2)] for i in range(2)]
    return d


def _variant_dict(c):
    return dict(block_m=c.block_m, block_n=c.block_n, block_k=c.block_k, waves_m=c.waves_m, waves_n=c.waves_n,
                mfma=c.mfma, stages=c.stages)


SHAPES = [(512, 512, 512), (4096, 4096, 4096), (8192, 8192, 8192), (1, 28672, 8192), (16, 8192, 28672),
          (256, 28672, 8192), (64, 64, 16384), (1808, 7344, 272), (11296, 64, 13504), (300, 520, 72), (16384, 16384, 64)]


@pytest.mark.parametrize("b_layout", [0, 1])
@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_shipped_model_terms_match_the_oracle(dtype, b_layout):
    from paper_2512_04226_amd import binding as g
    hw = _hw_dict(g)
    fields = ["n_mi", "l_mt_ideal", "l_compute", "occupancy", "tiles", "waves", "active_cu", "f_m", "f_n", "h_l2", "h_mall",
              "l_issue", "l_lds", "l_l2", "l_mall", "l_hbm", "l_mem", "l_mem_tail", "l_prologue", "l_epilogue",
              "l_iter", "iters", "l_tile", "l_tile_tail", "l_reduce", "l_total", "total_us"]
    checked = n_sk = 0
    for (M, N, K) in SHAPES:
        if dtype == 1 and (N % 16 or K % 16):
            continue
        for idx in range(g.gemm_cfg_count(dtype)):
            c = g.gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout)
            if c is None:
                continue
            assert c.b_layout == b_layout and c.ldb == (K if b_layout else N)
            p = g.gemm_predict(c)
            o = sm.predict(hw, dtype, M, N, K, _variant_dict(c), c.split_k, b_layout, c.stream_k)
            n_sk += c.stream_k
            for f in fields:
                assert getattr(p, f) == pytest.approx(o[f], rel=1e-9, abs=1e-9), (M, N, K, c.describe(), f)
            assert c.group_m == o["group_m"] and c.predicted_us == pytest.approx(o["total_us"], rel=1e-9)
            checked += 1
    assert checked > 500 and n_sk > 30


def test_pick_is_the_oracle_argmin():
    """gemm_select = first minimum of the oracle's predicted latency in enumeration order."""
    from paper_2512_04226_amd import binding as g
    hw = _hw_dict(g)
    for (M, N, K) in SHAPES:
        best = None
        for idx in range(g.gemm_cfg_count(0)):
            c = g.gemm_cfg_at(idx, M, N, K, 0)
            if c is None:
                continue
            t = sm.predict(hw, 0, M, N, K, _variant_dict(c), c.split_k, 0, c.stream_k)["l_total"]
            if best is None or t < best[0] * (1 - 1e-12):
                best = (t, c.kernel_id, c.split_k, c.stream_k)
        pick = g.gemm_select(M, N, K, 0)
        assert (pick.kernel_id, pick.split_k, pick.stream_k) == best[1:], (M, N, K, pick.describe())


@pytest.mark.parametrize("dtype", [0, 2])
def test_pick_on_k_contiguous_b_is_the_oracle_argmin_up_to_the_one_listed_tie(dtype):
    """On K-contiguous B the pick has the oracle's minimum latency; it is the first such entry in enumeration order unless
    that entry is the 4x2 wave grid of the 16-bit 256x256x64 tile (16x16x32 MFMA, two stages), whose exact tie with the 2x4
    grid of the same tile goes to the 2x4 grid on this layout (same split / Stream-K mode)."""
    from paper_2512_04226_amd import binding as g
    hw = _hw_dict(g)
    n_exception = 0
    for (M, N, K) in SHAPES:
        rows = []
        for idx in range(g.gemm_cfg_count(dtype)):
            c = g.gemm_cfg_at_ex(idx, M, N, K, dtype, 1)
            if c is None:
                continue
            t = sm.predict(hw, dtype, M, N, K, _variant_dict(c), c.split_k, 1, c.stream_k)["l_total"]
            rows.append((t, c))
        t_min = min(t for t, _ in rows)
        first = next(c for t, c in rows if t <= t_min * (1 + 1e-12))
        pick = g.gemm_select_ex(M, N, K, dtype, 1)
        t_pick = sm.predict(hw, dtype, M, N, K, _variant_dict(pick), pick.split_k, 1, pick.stream_k)["l_total"]
        assert t_pick == pytest.approx(t_min, rel=1e-12), (M, N, K, pick.describe())
        key = lambda c: (c.kernel_id, c.split_k, c.stream_k)
        if key(pick) != key(first):
            tile = lambda c: (c.block_m, c.block_n, c.block_k, c.mfma, c.stages, c.split_k, c.stream_k)
            assert tile(pick) == tile(first) == (256, 256, 64, 16, 2, first.split_k, first.stream_k), (M, N, K, pick.describe())
            assert (first.waves_m, first.waves_n) == (4, 2) and (pick.waves_m, pick.waves_n) == (2, 4)
            n_exception += 1
    assert n_exception >= 1      # 8192^3 and 4096^3 take the 2x4 grid


def test_retargeting_to_a_304_cu_table_changes_waves_cache_tiles_and_candidates():
    """Section I / V: the selector is ported by swapping the hardware table.  Under the 304-CU table
    Algorithm 4 must count waves of 304 tiles and Algorithm 6 must factor 38 CUs per L2; every
    shipped term must still agree with the oracle evaluated on that table."""
    from paper_2512_04226_amd import binding as g
    base = bytes(g.gemm_hw_get())
    try:
        g.gemm_hw_set(g.gemm_hw_preset(g.GEMM_HW_MI300X_LIKE))
        hw = _hw_dict(g)
        assert hw["n_cu"] == 304 and hw["n_xcd"] == 8 and hw["lds_bytes"] == 64 * 1024
        seen = 0
        for idx in range(g.gemm_cfg_count(0)):
            c = g.gemm_cfg_at(idx, 2432, 2048, 4096, 0)
            if c is None:
                continue
            # candidates must fit the smaller LDS
            assert c.stages * (c.block_m + c.block_n) * c.block_k * 2 <= 64 * 1024, c.describe()
            p = g.gemm_predict(c)
            o = sm.predict(hw, 0, 2432, 2048, 4096, _variant_dict(c), c.split_k, 0, c.stream_k)
            for f in ("tiles", "waves", "active_cu", "f_m", "f_n", "h_l2", "h_mall", "l_mem", "l_total"):
                assert getattr(p, f) == pytest.approx(o[f], rel=1e-9, abs=1e-9), (c.describe(), f)
            if (c.block_m, c.block_n, c.block_k, c.stages, c.split_k, c.stream_k) == (128, 128, 64, 2, 1, 0):
                # 19 x 16 = 304 tiles, one workgroup per CU (the ring fills the 64 KB LDS): exactly one full wave
                assert p.tiles == 304 and p.waves == 1 and p.active_cu == 304
                assert p.f_m * p.f_n == 38 and {p.f_m, p.f_n} == {2.0, 19.0}
                seen += 1
        assert seen >= 1
        pick_304 = g.gemm_select(2432, 2048, 4096, 0)
        assert pick_304.stages * (pick_304.block_m + pick_304.block_n) * pick_304.block_k * 2 <= 64 * 1024
    finally:
        g.gemm_hw_reset()
    assert bytes(g.gemm_hw_get()) == base
    p = g.gemm_predict(g.gemm_cfg_at(0, 4864, 4096, 4096, 0))
    assert p.waves == 2 and p.active_cu == 48
    with pytest.raises(g.GemmError):
        g.gemm_hw_preset(7)
    assert bytes(g.gemm_hw_preset(g.GEMM_HW_MI355X)) == base


def test_batched_selection_matches_the_oracle_and_scales_the_tile_count():
    """Algorithm 4 with a batch: `batch` times the tiles.  A batch of small problems fills the
    device, so the selector stops splitting K and may take larger tiles."""
    from paper_2512_04226_amd import binding as g
    hw = _hw_dict(g)
    M, N, K = 512, 512, 16384
    for batch in (1, 3, 64):
        best = None
        for idx in range(g.gemm_cfg_count(0)):
            c = g.gemm_cfg_at_batched(idx, M, N, K, batch, 0)
            if c is None:
                continue
            assert c.batch == batch and (c.stride_a, c.stride_b, c.stride_c) == (M * K, K * N, M * N)
            assert not (c.stream_k and batch > 1)
            p = g.gemm_predict(c)
            o = sm.predict(hw, 0, M, N, K, _variant_dict(c), c.split_k, 0, c.stream_k, batch)
            for f in ("tiles", "waves", "active_cu", "l_reduce", "l_tile", "l_total", "total_us"):
                assert getattr(p, f) == pytest.approx(o[f], rel=1e-9, abs=1e-9), (batch, c.describe(), f)
            tiles_1 = -(-M // c.block_m) * -(-N // c.block_n) * c.split_k
            assert p.tiles == tiles_1 * batch
            if best is None or o["l_total"] < best[0] * (1 - 1e-12):
                best = (o["l_total"], c.kernel_id, c.split_k, c.stream_k)
        pick = g.gemm_select_batched(M, N, K, batch, 0)
        assert (pick.kernel_id, pick.split_k, pick.stream_k) == best[1:]
    one, many = g.gemm_select_batched(M, N, K, 1, 0), g.gemm_select_batched(M, N, K, 64, 0)
    assert one.split_k > 1 and many.split_k == 1
    assert many.block_m * many.block_n >= one.block_m * one.block_n
    assert g.gemm_workspace_bytes(one) == one.split_k * M * N * 4
    with pytest.raises(g.GemmError):
        g.gemm_select_batched(M, N, K, 0, 0)
    with pytest.raises(g.GemmError):
        g.gemm_select_batched(M, N, K, 70000, 0)
