"""Hand-worked examples of the selector's model (tests/golden/model_worked_examples.json) against
(a) the checker in oracle/ and (b) the library, separately: neither is the other's reference, both must
reproduce literal numbers whose arithmetic is written out in the fixture.  Plus the reductions and
properties that tie the composed model back to the paper's printed algorithms."""
import json
import os

import pytest

from oracle import selector_model as sm

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "model_worked_examples.json")))
REL = 1e-9


def _hw(example):
    hw = dict(GOLD["hw"])
    hw.update(example.get("hw_override", {}))
    return hw


def _close(got, want):
    return got == pytest.approx(want, rel=REL, abs=1e-9)


# ------------------------------------------------------------------ (a) the checker against the literals

@pytest.mark.parametrize("ex", GOLD["examples"], ids=lambda e: e["name"].split()[0])
def test_checker_reproduces_the_worked_examples(ex):
    out = sm.predict(_hw(ex), ex["dtype"], ex["M"], ex["N"], ex["K"], ex["variant"], ex["split_k"], ex["b_layout"],
                     ex["stream_k"])
    for field, want in ex["expect"].items():
        assert _close(out[field], want), (ex["name"], field, out[field], want)


@pytest.mark.parametrize("ex", GOLD["grouped"], ids=lambda e: e["name"].split()[0])
def test_checker_reproduces_the_grouped_example(ex):
    total, bands = sm.predict_grouped(_hw(ex), ex["dtype"], [tuple(s) for s in ex["shapes"]], ex["variant"], ex["b_layout"])
    assert _close(total, ex["expect"]["l_total"]) and bands == ex["expect"]["group_m"]


def test_checker_functions_reproduce_their_examples():
    hw = dict(GOLD["hw"])
    f = GOLD["functions"]
    for case in f["resident_workgroups"]:
        assert sm.resident_workgroups(hw, case["variant"], case["es"]) == case["expect"], case["why"]
    for seg, want in f["segment_efficiency"]:
        assert _close(sm.segment_efficiency(hw, seg), want), seg
    for case in f["split_k_reduce"]:
        assert _close(sm.split_k_reduce(hw, case["M"], case["N"], case["split_k"], case["batch"]), case["expect"]), case["why"]
    for case in f["stream_k_sum"]:
        assert _close(sm.stream_k_sum(hw, case["variant"], case["slots"], case["left"]), case["expect"]), case["why"]
    for case in f["wave_split"]:
        assert list(sm.wave_split(case["tiles"], case["n_cu"], case["occ"])) == case["expect"], case
    for case in f["level_times_hbm"]:
        got = sm.level_times(hw, case["variant"], case["es"], case["b_layout"], case["tiles_per_cu"], case["active_cus"],
                             case["h_first"], case["h_second"], case["rows_valid"], case["cols_valid"],
                             one_tile_row=case["one_tile_row"])["l_hbm"]
        assert _close(got, case["expect"]), case["why"]


# ------------------------------------------------------------------ (b) the library against the same literals

def _lib_hw(g, hw):
    h = g.gemm_hw_get()
    for name, value in hw.items():
        if name == "l_mi_clk":
            for i in range(2):
                for j in range(2):
                    h.l_mi_clk[i][j] = value[i][j]
        else:
            setattr(h, name, type(getattr(h, name))(value))
    return h


def _lib_cfg(g, ex):
    v = ex["variant"]
    for idx in range(g.gemm_cfg_count(ex["dtype"])):
        c = g.gemm_cfg_at_ex(idx, ex["M"], ex["N"], ex["K"], ex["dtype"], ex["b_layout"])
        if c is not None and (c.block_m, c.block_n, c.block_k, c.waves_m, c.waves_n, c.mfma, c.stages, c.split_k,
                              c.stream_k) == (v["block_m"], v["block_n"], v["block_k"], v["waves_m"], v["waves_n"],
                                              v["mfma"], v["stages"], ex["split_k"], ex["stream_k"]):
            return c
    raise AssertionError("the library has no such configuration: %s" % ex["name"])


@pytest.mark.parametrize("ex", GOLD["examples"], ids=lambda e: e["name"].split()[0])
def test_library_reproduces_the_worked_examples(ex):
    from paper_2512_04226_amd import binding as g
    try:
        g.gemm_hw_set(_lib_hw(g, _hw(ex)))
        cfg = _lib_cfg(g, ex)
        p = g.gemm_predict(cfg)
        for field, want in ex["expect"].items():
            got = cfg.group_m if field == "group_m" else getattr(p, field)
            assert _close(got, want), (ex["name"], field, got, want)
        if "total_us" in ex["expect"]:
            assert _close(cfg.predicted_us, ex["expect"]["total_us"])
    finally:
        g.gemm_hw_reset()


@pytest.mark.parametrize("ex", GOLD["grouped"], ids=lambda e: e["name"].split()[0])
def test_library_reproduces_the_grouped_example(ex):
    from paper_2512_04226_amd import binding as g
    try:
        hw = _hw(ex)
        g.gemm_hw_set(_lib_hw(g, hw))
        shapes = [tuple(s) for s in ex["shapes"]]
        probs = g.make_problems(shapes, ex["b_layout"])
        v = ex["variant"]
        hit = None
        for vid in range(g.gemm_variant_count(ex["dtype"])):
            c = g.gemm_cfg_at_grouped(vid, probs, ex["dtype"], ex["b_layout"])
            if c is not None and (c.block_m, c.block_n, c.block_k, c.waves_m, c.waves_n, c.mfma, c.stages) == (
                    v["block_m"], v["block_n"], v["block_k"], v["waves_m"], v["waves_n"], v["mfma"], v["stages"]):
                hit = c
        assert hit is not None
        assert _close(hit.predicted_us, ex["expect"]["l_total"] / (hw["clk_ghz"] * 1e3))
        for i, pr in enumerate(probs):          # the plan validates pointers it never follows: any aligned address
            pr.A, pr.B, pr.C = 0x10000 * (3 * i + 1), 0x10000 * (3 * i + 2), 0x10000 * (3 * i + 3)
        table, _ = g.gemm_grouped_plan(hit, probs)
        by_k = {(r.M, r.N, r.K): r.group_m for r in table}
        assert [by_k[s] for s in shapes] == ex["expect"]["group_m"]
    finally:
        g.gemm_hw_reset()


# ------------------------------------------------------------------ reductions to the printed algorithms

def _plain_hw(**over):
    """A table on which every reading that adds to the paper's formulas is switched off."""
    hw = dict(n_cu=256, n_xcd=8, simd_per_cu=4, lds_bytes=160 * 1024, l2_bytes=4 << 20, mall_bytes=256 << 20, clk_ghz=2.4,
              hbm_bytes_per_clk=2500.0, mall_bytes_per_clk=6000.0, l2_bytes_per_clk=2048.0, lds_bytes_per_clk=1e18,
              lds_tr_bytes_per_clk=1e18, vmem_bytes_per_clk=64.0, mem_latency_clk=700.0, cache_eff_frac=1.0, launch_clk=0.0,
              wg_overhead_clk=0.0, epilogue_clk=0.0, reduce_launch_clk=0.0, under_occ_frac=1.0, seg_eff_lo=1.0,
              overlap_frac=0.0, l_mi_clk=[[32.0, 16.0], [64.0, 32.0]], fill_issue_bytes_per_clk=1e18, slab_sync_clk=0.0)
    hw.update(over)
    return hw


def test_level_times_is_algorithm_7_when_the_added_terms_are_off():
    """One workgroup per CU, a two-stage ring (so the whole latency is paid per iteration), perfect row
    segments, an LDS that costs nothing: the printed product form of the HBM share gives Algorithm 7
    exactly; the nested-scope reading differs from it in the HBM term only."""
    hw = _plain_hw()
    v = dict(block_m=256, block_n=128, block_k=64, waves_m=2, waves_n=2, mfma=32, stages=2)
    for (c, h1, h2) in ((256.0, 0.8125, 0.9375), (40.0, 0.3, 0.1), (256.0, 0.0, 0.0), (7.0, 0.9, 0.95)):
        ld_cu = (v["block_m"] + v["block_n"]) * v["block_k"] * 2
        want = sm.alg7_memory_latency(ld_cu, c, h1, h2, hw["vmem_bytes_per_clk"], hw["l2_bytes_per_clk"] * min(8.0, c),
                                      hw["mall_bytes_per_clk"], hw["hbm_bytes_per_clk"], hw["mem_latency_clk"])
        got = sm.level_times(hw, v, 2, 0, 1.0, c, h1, h2, v["block_m"], v["block_n"], hbm_share="product")
        assert _close(got["l_mem"], want)
        assert _close(got["l_issue"], ld_cu / 64.0) and got["l_lds"] < 1e-9
        nested = sm.level_times(hw, v, 2, 0, 1.0, c, h1, h2, v["block_m"], v["block_n"])
        for term in ("l_issue", "l_lds", "l_l2", "l_mall"):
            assert nested[term] == got[term]
        assert _close(nested["l_hbm"] - 700.0, min(1 - h1, 1 - h2) * ld_cu * c / 2500.0)
        assert _close(got["l_hbm"] - 700.0, (1 - h1) * (1 - h2) * ld_cu * c / 2500.0)
        assert nested["l_hbm"] >= got["l_hbm"] - 1e-12


def test_composition_is_algorithms_8_and_9_when_the_added_terms_are_off():
    """Full waves of one workgroup per CU and no fixed costs: the composed total is Algorithm 9 applied to
    Algorithm 8's tile latency (with the one extra drain term), computed here from the printed functions and
    the problem's numbers alone -- nothing of the composed model's output is fed back in."""
    hw = _plain_hw(mem_latency_clk=0.0)
    v = dict(block_m=256, block_n=256, block_k=64, waves_m=2, waves_n=2, mfma=32, stages=2)
    M = N = K = 8192
    n_mi, l_mt = sm.alg3_compute_latency(32, 32, 16, 256, 256, 64, 32.0)
    l_comp = l_mt / 4
    h1, h2 = sm.alg5_hit_rate(4, 8, 256, 256, 64), sm.alg5_hit_rate(16, 16, 256, 256, 64)
    ld_cu = 512 * 64 * 2
    l_mem = max(ld_cu / 64.0, ld_cu * 256 / (8 * 2048.0), (1 - h1) * ld_cu * 256 / 6000.0,
                min(1 - h1, 1 - h2) * ld_cu * 256 / 2500.0)
    out_elems = 256 * 256 * 256                    # all active tiles' outputs, two bytes each, through the HBM rate
    l_tile = sm.alg8_tile_latency(K, 64, l_mem, l_comp, 2, out_elems, 1, 2500.0) + l_comp
    o = sm.predict(hw, 0, M, N, K, v, 1)
    assert o["n_mi"] == n_mi and _close(o["l_compute"], l_comp) and _close(o["l_mem"], l_mem)
    assert _close(o["l_tile"], l_tile)
    assert _close(o["l_total"], sm.alg9_total_latency(M, N, 256, 256, 256, l_tile))
    # and the library on the same table
    from paper_2512_04226_amd import binding as g
    try:
        g.gemm_hw_set(_lib_hw(g, hw))
        cfg = _lib_cfg(g, dict(variant=v, dtype=0, b_layout=0, M=M, N=N, K=K, split_k=1, stream_k=0, name="plain"))
        p = g.gemm_predict(cfg)
        assert _close(p.l_tile, l_tile) and _close(p.l_total, sm.alg9_total_latency(M, N, 256, 256, 256, l_tile))
    finally:
        g.gemm_hw_reset()


RATES = ("hbm_bytes_per_clk", "mall_bytes_per_clk", "l2_bytes_per_clk", "lds_bytes_per_clk", "lds_tr_bytes_per_clk",
         "vmem_bytes_per_clk", "fill_issue_bytes_per_clk")
COSTS = ("mem_latency_clk", "launch_clk", "wg_overhead_clk", "epilogue_clk", "reduce_launch_clk", "slab_sync_clk")
SHAPES = [(8192, 8192, 8192, 1, 0), (200, 1000, 4096, 4, 0), (16, 28672, 8192, 1, 0), (4352, 4096, 4096, 1, 1), (4096, 4096, 128, 1, 0)]


@pytest.mark.parametrize("side", ["checker", "library"])
def test_latency_is_monotone_in_every_rate_and_cost(side):
    """A faster level never makes a prediction slower, a larger fixed cost never makes it faster (a dropped
    term, a rate multiplied instead of divided, or a sign error breaks this for some field)."""
    from paper_2512_04226_amd import binding as g
    base = dict(GOLD["hw"])
    variants = [GOLD["examples"][0]["variant"], GOLD["examples"][3]["variant"],
                dict(block_m=16, block_n=128, block_k=128, waves_m=1, waves_n=4, mfma=16, stages=4)]

    def total(hw, v, M, N, K, split, sk):
        if side == "checker":
            if sk and sm.stream_k_split(-(-M // v["block_m"]) * -(-N // v["block_n"]),
                                        hw["n_cu"] * sm.resident_workgroups(hw, v, 2), -(-K // v["block_k"])) is None:
                return None
            return sm.predict(hw, 0, M, N, K, v, split, 0, sk)["l_total"]
        g.gemm_hw_set(_lib_hw(g, hw))
        try:
            cfg = _lib_cfg(g, dict(variant=v, dtype=0, b_layout=0, M=M, N=N, K=K, split_k=split, stream_k=sk, name="m"))
        except AssertionError:
            return None
        return g.gemm_predict(cfg).l_total

    try:
        checked = 0
        for v in variants:
            for (M, N, K, split, sk) in SHAPES:
                t0 = total(base, v, M, N, K, split, sk)
                if t0 is None:
                    continue
                for name in RATES + COSTS:
                    t1 = total(dict(base, **{name: base[name] * 1.5}), v, M, N, K, split, sk)
                    if name in RATES:
                        assert t1 <= t0 * (1 + 1e-12), (name, v, M, N, K)
                    else:
                        assert t1 >= t0 * (1 - 1e-12), (name, v, M, N, K)
                    checked += 1
        assert checked >= 100
    finally:
        g.gemm_hw_reset()


def test_the_compute_term_carries_no_per_kernel_timing():
    """Two variants with the same tile, wave count and matrix instruction are priced alike whatever their ring
    depth; a variant's compute latency follows from Algorithm 3's count and the descriptor alone."""
    hw = dict(GOLD["hw"])
    a = dict(block_m=128, block_n=128, block_k=64, waves_m=2, waves_n=4, mfma=16, stages=3)
    b = dict(a, stages=4)
    assert sm.slab_compute(hw, a, 0) == sm.slab_compute(hw, b, 0)
    n_mi, l_mt, cost = sm.slab_compute(hw, a, 0)
    assert n_mi == 8 * 8 * 2 and l_mt == 128 * 20.0 / 4 and cost == l_mt + 256 * 64 * 2 / 64.0 + 100.0
    # doubling every issue interval doubles L_MT and nothing else
    slow = dict(hw, l_mi_clk=[[80.0, 40.0], [160.0, 80.0]])
    assert sm.slab_compute(slow, a, 0)[2] - cost == l_mt
