"""Checker for the analytical selector (TEST INFRASTRUCTURE ONLY: nothing under the product package
imports this module, and it shares no code, table or constant with it).

Two layers.

1. The paper's Section IV as printed, one small function per algorithm (`alg3_...` to `alg9_...`):
   instruction count and latency of a workgroup tile (Algorithm 3), output tiles / waves / remainder
   (Algorithm 4), cache-tile hit rate (Algorithm 5), factor pairs of a CU count (Algorithm 6), memory
   latency of one loop iteration as a maximum over the levels of the hierarchy (Algorithm 7), latency of
   one output tile (Algorithm 8) and of the whole product (Algorithm 9).  They are pinned to the values
   and closed forms the paper fixes (tests/test_selector_model.py, tests/golden/paper_worked_examples.txt).

2. The model the library is specified to evaluate: the same algorithms with the readings that fill in what
   the paper leaves open.  Every reading is a function of its own with the reading stated in its docstring
   (`resident_workgroups`, `wave_split`, `cache_tile`, `derate`, `segment_efficiency`, `slab_compute`,
   `level_times`, `tile_time`, `split_k_reduce`, `stream_k_phase`, `stream_k_sum`), `predict` and
   `predict_grouped` put them together.  Each is pinned to hand-worked examples whose arithmetic is written
   out in tests/golden/model_worked_examples.json; the library is checked against the same literal numbers
   separately, so neither side is the other's reference.

Units: bytes and compute clocks.  `hw` is a dict with the fields of the hardware descriptor; a variant `v`
is a dict with block_m, block_n, block_k, waves_m, waves_n, mfma (32 or 16) and stages.
"""
import math

# ------------------------------------------------------------------ Section IV as printed


def alg3_compute_latency(mi_m, mi_n, mi_k, mt_m, mt_n, mt_k, l_mi):
    """Algorithm 3.  A workgroup tile is covered by whole matrix instructions along each of its three
    extents; its latency is the instruction count times one instruction's latency.  -> (N_MI, L_MT)"""
    count = 1
    for extent, step in ((mt_m, mi_m), (mt_n, mi_n), (mt_k, mi_k)):
        count *= -(-extent // step)
    return count, count * l_mi


def alg4_occupancy(M, N, mt_m, mt_n, n_cu):
    """Algorithm 4 exactly as printed: (T_out mod N_CU, waves, T_out).  The remainder is 0 when the last
    wave is full -- also in the paper's own one-tile-per-CU example."""
    t_out = (-(-M // mt_m)) * (-(-N // mt_n))
    return t_out % n_cu, -(-t_out // n_cu), t_out


def alg5_hit_rate(m_t, n_t, M_T, N_T, K_T):
    """Algorithm 5.  An m_t x n_t block of workgroup tiles requests m_t*n_t*(M_T + N_T)*K_T operand
    elements per K step, of which only the m_t row panels and n_t column panels are distinct."""
    distinct = (m_t * M_T + n_t * N_T) * K_T
    requested = m_t * n_t * (M_T + N_T) * K_T
    return 1 - distinct / requested


def alg6_factorizations(n_cu_cache):
    """Algorithm 6: the ordered pairs (f_m, f_n) with f_m * f_n = N_CU_cache, ascending f_m."""
    return [(d, n_cu_cache // d) for d in range(1, n_cu_cache + 1) if n_cu_cache % d == 0]


def alg7_memory_latency(ld_cu, C, H1, H2, R_L1, R_1, R_2, R_MEM, L_lat):
    """Algorithm 7 as printed.  Every CU issues its own loads at R_L1; all C CUs' traffic goes through
    the first shared level at R_1; what misses it (1 - H1) goes through the second at R_2; what misses
    that too (1 - H2 of the rest) comes from memory at R_MEM after a latency L_lat.  The slowest of
    these is the iteration's memory latency."""
    everything = ld_cu * C
    past_first = (1 - H1) * everything
    past_second = (1 - H2) * past_first
    return max(ld_cu / R_L1, everything / R_1, past_first / R_2, past_second / R_MEM + L_lat)


def alg8_tile_latency(K, k_t, l_mem, l_compute, a, m_t, n_t, R_mem):
    """Algorithm 8 as printed: one load (prologue), a store of a * m_t * n_t output elements (epilogue),
    and ceil(K / k_t) - 1 iterations in which loading and computing overlap."""
    iterations = -(-K // k_t) - 1
    return l_mem + a * m_t * n_t / R_mem + iterations * max(l_compute, l_mem)


def alg9_total_latency(M, N, m_t, n_t, n_cu, l_tile):
    """Algorithm 9 as printed: waves of N_CU output tiles, each as long as one tile."""
    return alg4_occupancy(M, N, m_t, n_t, n_cu)[1] * l_tile


# ------------------------------------------------------------------ the readings, one function each


def _elem_bytes(dtype):
    return 1 if dtype == 1 else 2          # dtype 0 bf16, 1 fp8 e4m3, 2 fp16


def _mfma_k(dtype, mfma):
    """K extent of the matrix instruction: 16-bit 32x32x16 / 16x16x32, fp8 32x32x64 / 16x16x128."""
    return (64 if mfma == 32 else 128) if dtype == 1 else (16 if mfma == 32 else 32)


def resident_workgroups(hw, v, es):
    """READING (not in the paper, which has one workgroup per CU): several workgroups of a small variant
    share a CU.  How many: what fits the LDS (the ring of `stages` slabs), what fits the 512 registers a
    SIMD lane offers its waves (fp32 accumulators of the tile spread over the lanes, plus 64 for fragments
    and addresses; at most 8 waves per SIMD), never more than 8 and never fewer than 1."""
    ring = v["stages"] * (v["block_m"] + v["block_n"]) * v["block_k"] * es
    waves_per_wg = v["waves_m"] * v["waves_n"]
    regs_per_lane = v["block_m"] * v["block_n"] / (64.0 * waves_per_wg) + 64.0
    waves_per_simd = min(8, max(1, int(512.0 // regs_per_lane)))
    fit_regs = waves_per_simd * hw["simd_per_cu"] // waves_per_wg
    fit_lds = int(hw["lds_bytes"] // ring)
    return max(1, min(fit_regs, fit_lds, 8))


occupancy = resident_workgroups


def wave_split(tiles, n_cu, occ):
    """READING of Algorithm 4: a wave is n_cu * occ workgroup slots; the last wave holds what is left, and a
    remainder of zero means a FULL last wave (the printed modulo would make it empty).  In the last wave
    the tiles spread over as many CUs as there are tiles (at most all), ceil(tail / n_cu) to a CU.
    -> (waves, tail tiles, active CUs, tiles per CU in the tail)"""
    slots = n_cu * occ
    waves = -(-tiles // slots)
    tail = tiles - (waves - 1) * slots
    return waves, tail, min(tail, n_cu), -(-tail // n_cu)


def cache_tile(scope, v, tiles_m, tiles_n):
    """READING of Algorithm 6's choice (its floor(sqrt(N)) default is not a divisor of 32): of all factor
    pairs of the scope's workgroup count, each clipped to the tile grid, the one with the highest
    Algorithm-5 hit rate for this variant's nominal tile; between equal rates the cache tile closer to
    square in elements, then the wider one, else the earlier pair.  -> (f_m, f_n, unclipped f_m)"""
    ranked = []
    for order, (i, j) in enumerate(alg6_factorizations(scope)):
        f_m, f_n = min(i, tiles_m), min(j, tiles_n)
        rate = min(1.0, max(0.0, alg5_hit_rate(f_m, f_n, v["block_m"], v["block_n"], v["block_k"])))
        ranked.append((rate, -abs(f_m * v["block_m"] - f_n * v["block_n"]), f_n, -order, f_m, i))
    # exact ties are ties here: the candidates' rates and skews are small rationals
    top = max(ranked, key=lambda c: (round(c[0], 12), round(c[1], 9), c[2], c[3]))
    return top[4], top[2], top[5]


def derate(hit, f_m, f_n, v, es, capacity, usable_share):
    """READING of Section IV-C's capacity remark (no formula given): the cache tile's working set of one K
    step, two slabs deep, against the usable share of the cache; beyond it the hit rate shrinks in
    proportion."""
    working_set = (f_m * v["block_m"] + f_n * v["block_n"]) * v["block_k"] * es * 2.0
    return hit * min(1.0, usable_share * capacity / working_set)


def segment_efficiency(hw, seg):
    """READING (not in the paper): share of the HBM rate reached when a tile touches `seg` contiguous bytes
    of each matrix row: all of it from 256 bytes up, seg_eff_lo at 32 bytes and below, linear in log2 between."""
    if seg >= 256:
        return 1.0
    octaves = math.log2(max(seg, 32.0) / 32.0)          # 0 .. 3
    return min(1.0, hw["seg_eff_lo"] + (1.0 - hw["seg_eff_lo"]) * octaves / 3.0)


def slab_compute(hw, v, dtype):
    """READING of Algorithm 3's use in Algorithm 8.  (N_MI, L_MT spread over the SIMDs the workgroup's
    waves occupy, compute latency of one K slab of one tile).  The last is L_MT plus what the slab's fill and
    its barrier take out of the waves' instruction streams: the (BM + BN) * BK bytes of the slab are loaded
    by the same waves, in order with their matrix instructions, at fill_issue_bytes_per_clk, and every slab
    ends in one synchronisation of slab_sync_clk.  L_MI is the issue interval the chip sustains on
    workload-like operands (it is power-limited), one per instruction shape."""
    es = _elem_bytes(dtype)
    row = 1 if dtype == 1 else 0                          # fp16 runs at bf16's rates
    l_mi = hw["l_mi_clk"][row][0 if v["mfma"] == 32 else 1]
    n_mi, l_mt = alg3_compute_latency(v["mfma"], v["mfma"], _mfma_k(dtype, v["mfma"]),
                                      v["block_m"], v["block_n"], v["block_k"], l_mi)
    l_mt_spread = l_mt / min(hw["simd_per_cu"], v["waves_m"] * v["waves_n"])
    fill = (v["block_m"] + v["block_n"]) * v["block_k"] * es
    return n_mi, l_mt_spread, l_mt_spread + fill / hw["fill_issue_bytes_per_clk"] + hw["slab_sync_clk"]


def level_times(hw, v, es, b_layout, tiles_per_cu, active_cus, h_first, h_second, rows_valid, cols_valid,
                tiles_per_cu_moving=None, hbm_share="neither", one_tile_row=False):
    """Algorithm 7 in bytes and clocks for one K step, with these READINGS:
    * Ld_CU (undefined in the paper) is the slab of every tile a CU works on: the load INSTRUCTIONS cover the
      nominal (BM + BN) * BK elements, the BYTES that move only the valid rows and columns of the tile
      (`rows_valid` x `cols_valid`, the mean over the tile grid) of `tiles_per_cu_moving` tiles;
    * first shared level = the L2 of one XCD (traffic divides over the XCDs that have work), second = MALL;
    * an LDS term joins the maximum (Section IV-D lists the bound, Algorithm 7 omits it): every wave reads its
      rows of A and its columns of B from LDS, so A's slab is read waves_n times and B's waves_m times, B at
      the transpose-read rate unless it is stored K-contiguous;
    * the share of requested bytes that reaches HBM is what NEITHER cache holds, min(1 - H1, 1 - H2), because
      the two rates come from nested scopes (hbm_share="product" gives the printed (1 - H1)(1 - H2));
    * each operand's HBM bytes are divided by its row-segment efficiency (K-contiguous B under a grid of one tile
      row: every piece of a row is read once, by one workgroup, whose next slab continues the row, so the piece
      counts twice);
    * the latency is shared by the slabs in flight: L_lat / max(1, tiles_per_cu * (stages - 1)).
    -> dict of the five terms and their maximum."""
    moving = tiles_per_cu if tiles_per_cu_moving is None else tiles_per_cu_moving
    slab_k_bytes = v["block_k"] * es
    issue = (v["block_m"] + v["block_n"]) * slab_k_bytes * tiles_per_cu / hw["vmem_bytes_per_clk"]
    a_moved = rows_valid * slab_k_bytes * moving
    b_moved = cols_valid * slab_k_bytes * moving
    b_read_rate = hw["lds_bytes_per_clk"] if b_layout else hw["lds_tr_bytes_per_clk"]
    lds = tiles_per_cu * (v["block_m"] * v["waves_n"] * slab_k_bytes / hw["lds_bytes_per_clk"]
                          + v["block_n"] * v["waves_m"] * slab_k_bytes / b_read_rate)
    device_bytes = (a_moved + b_moved) * active_cus
    l2 = device_bytes / min(hw["n_xcd"], max(1.0, active_cus)) / hw["l2_bytes_per_clk"]
    mall = (1.0 - h_first) * device_bytes / hw["mall_bytes_per_clk"]
    if hbm_share == "product":
        miss_both = (1.0 - h_first) * (1.0 - h_second)
    else:
        miss_both = min(1.0 - h_first, 1.0 - h_second)
    seg_a = segment_efficiency(hw, slab_k_bytes)
    seg_b = segment_efficiency(hw, ((2 if one_tile_row else 1) * v["block_k"] if b_layout else v["block_n"]) * es)
    hbm = (miss_both * (a_moved / seg_a + b_moved / seg_b) * active_cus / hw["hbm_bytes_per_clk"]
           + hw["mem_latency_clk"] / max(1.0, tiles_per_cu * (v["stages"] - 1)))
    return {"l_issue": issue, "l_lds": lds, "l_l2": l2, "l_mall": mall, "l_hbm": hbm,
            "l_mem": max(issue, lds, l2, mall, hbm)}


def tile_time(hw, v, slab_cost, occ, tiles_per_cu, active_cus, slabs, out_bytes, mem):
    """Algorithm 8 with these READINGS: the compute latency of a K step is `slab_cost` per resident tile (a
    CU that holds fewer tiles than fit runs each a little faster: factor u + (1 - u) * held / fit with
    u = under_occ_frac); the prologue also pays the full memory latency and a per-workgroup cost; the
    epilogue moves the output bytes of all active tiles through the HBM rate plus a fixed cost; the last
    slab's compute is exposed (Algorithm 8 stops at ceil(K / k_t) - 1 iterations and never computes it)."""
    compute = slab_cost * tiles_per_cu
    if tiles_per_cu < occ:
        compute *= hw["under_occ_frac"] + (1.0 - hw["under_occ_frac"]) * tiles_per_cu / occ
    prologue = mem["l_mem"] + hw["mem_latency_clk"] + hw["wg_overhead_clk"]
    epilogue = (active_cus * tiles_per_cu * v["block_m"] * v["block_n"] * out_bytes / hw["hbm_bytes_per_clk"]
                + hw["epilogue_clk"])
    iteration = max(compute, mem["l_mem"])
    return {"l_compute": compute, "l_prologue": prologue, "l_epilogue": epilogue, "l_iter": iteration,
            "l_tile": prologue + epilogue + iteration * (slabs - 1) + compute}


def split_k_reduce(hw, M, N, split_k, batch=1):
    """READING of Section IV-D's "unroll the K loop" across CUs: the slices leave fp32 partial sums
    (split_k * M * N * 4 bytes) that a second launch reads and turns into M * N 16-bit outputs; that
    traffic runs at the MALL rate while it fits the usable share of the MALL, else at the HBM rate."""
    if split_k <= 1:
        return 0.0
    traffic = M * N * (4.0 * split_k + 2.0) * batch
    fits = traffic <= hw["cache_eff_frac"] * hw["mall_bytes"]
    return hw["reduce_launch_clk"] + traffic / (hw["mall_bytes_per_clk"] if fits else hw["hbm_bytes_per_clk"])


def stream_k_split(tiles, slots, slabs):
    """Hybrid Stream-K (Section V-E names Stream-K; READING: whole waves stay one tile per workgroup, the
    tiles % slots left over are cut along K into one equal range per slot).  -> (whole waves, stream-K
    tiles, slabs per worker), or None when nothing is left over or there are fewer slabs than workers."""
    left = tiles % slots
    if left == 0 or left * slabs < slots:
        return None
    return (tiles - left) // slots, left, left * slabs / slots


def stream_k_phase(hw, v, occ, slots, left, per_worker, slab_cost_full, mem_no_l2):
    """READING: the Stream-K phase keeps every CU full; its workers sit at different K offsets of different
    tiles, so it is priced with an L2 hit rate of zero (`mem_no_l2`); every worker stores one fp32 partial
    tile and the share left / slots of them, which straddle two tiles, pays prologue and store twice."""
    iteration = max(slab_cost_full, mem_no_l2["l_mem"])
    prologue = mem_no_l2["l_mem"] + hw["mem_latency_clk"] + hw["wg_overhead_clk"]
    store = hw["n_cu"] * occ * v["block_m"] * v["block_n"] * 4.0 / hw["hbm_bytes_per_clk"] + hw["epilogue_clk"]
    return (1.0 + left / slots) * (prologue + store) + iteration * (per_worker - 1.0) + slab_cost_full


def stream_k_sum(hw, v, slots, left):
    """READING: the summation pass reads slots + left fp32 partial tiles and writes left 16-bit tiles (MALL
    rate while that fits its usable share, else HBM), after a second launch, and one output's contributors
    (floor(slots / left) + 2 at most) form a dependent chain shared by 1, 4 or 8 thread rows (more than 8
    contributors: 4 rows; more than 32: 8) with four loads in flight each."""
    tile_elems = v["block_m"] * v["block_n"]
    traffic = (slots + left) * tile_elems * 4.0 + left * tile_elems * 2.0
    fits = traffic <= hw["cache_eff_frac"] * hw["mall_bytes"]
    contributors = slots // left + 2
    rows = 8 if contributors > 32 else 4 if contributors > 8 else 1
    chain = math.ceil(contributors / (4.0 * rows)) * hw["mem_latency_clk"]
    return hw["reduce_launch_clk"] + traffic / (hw["mall_bytes_per_clk"] if fits else hw["hbm_bytes_per_clk"]) + chain


# ------------------------------------------------------------------ composition


def predict(hw, dtype, M, N, K, v, split_k, b_layout=0, stream_k=0, batch=1):
    """All model terms for one configuration (names as in the C ABI's gemm_prediction, plus group_m,
    occupancy and l_tile_full).  READINGS made here: K slices and batch members count as tiles in Algorithm 4;
    hit rates are evaluated on the mean valid extent of a tile; Algorithm 9 prices the full waves and the
    last wave separately, adds one launch, and, with two or more workgroups resident per CU, lets a share
    overlap_frac of a tile's prologue and store stage hide under the other workgroups' K loops in every
    wave that another wave follows."""
    es = _elem_bytes(dtype)
    out = {}
    out["n_mi"], out["l_mt_ideal"], slab_cost = slab_compute(hw, v, dtype)

    tiles_m, tiles_n = -(-M // v["block_m"]), -(-N // v["block_n"])
    occ = resident_workgroups(hw, v, es)
    tiles = tiles_m * tiles_n * split_k * batch
    waves, tail, active, tail_per_cu = wave_split(tiles, hw["n_cu"], occ)
    out.update(tiles=tiles, waves=waves, active_cu=active, occupancy=occ)

    rows_valid, cols_valid = M / tiles_m, N / tiles_n
    hits = []
    for scope, capacity in ((hw["n_cu"] // hw["n_xcd"] * occ, hw["l2_bytes"]), (hw["n_cu"] * occ, hw["mall_bytes"])):
        f_m, f_n, raw = cache_tile(scope, v, tiles_m, tiles_n)
        rate = min(1.0, max(0.0, alg5_hit_rate(f_m, f_n, rows_valid, cols_valid, v["block_k"])))
        hits.append((derate(rate, f_m, f_n, v, es, capacity, hw["cache_eff_frac"]), f_m, f_n, raw))
    (h1, f_m1, f_n1, raw1), (h2, _, _, _) = hits
    out.update(f_m=f_m1, f_n=f_n1, h_l2=h1, h_mall=h2, group_m=max(1, min(raw1, tiles_m)))

    slabs = -(-(-(-K // v["block_k"])) // split_k)        # K slabs of one slice
    out["iters"] = slabs - 1
    out_bytes = 4.0 if split_k > 1 else 2.0

    def wave(tiles_per_cu, active_cus, moving=None, h_first=h1):
        mem = level_times(hw, v, es, b_layout, tiles_per_cu, active_cus, h_first, h2, rows_valid, cols_valid, moving,
                          one_tile_row=tiles_m == 1)
        return dict(mem, **tile_time(hw, v, slab_cost, occ, tiles_per_cu, active_cus, slabs, out_bytes, mem))

    full = wave(float(occ), float(hw["n_cu"]))
    last = wave(float(tail_per_cu), float(active), tail / active)    # the last wave moves the bytes of the tiles that exist
    reported = full if waves > 1 else last
    for name in ("l_compute", "l_issue", "l_lds", "l_l2", "l_mall", "l_hbm", "l_mem", "l_prologue", "l_epilogue",
                 "l_iter", "l_tile"):
        out[name] = reported[name]
    out.update(l_mem_tail=last["l_mem"], l_tile_tail=last["l_tile"], l_tile_full=full["l_tile"])

    out["l_reduce"] = split_k_reduce(hw, M, N, split_k, batch)
    hidden = hw["overlap_frac"] * (full["l_prologue"] + full["l_epilogue"]) if (occ >= 2 and waves > 1) else 0.0
    out["l_total"] = hw["launch_clk"] + (waves - 1) * (full["l_tile"] - hidden) + last["l_tile"] + out["l_reduce"]

    if stream_k:
        slots = hw["n_cu"] * occ
        whole, left, per_worker = stream_k_split(tiles, slots, slabs)
        no_l2 = level_times(hw, v, es, b_layout, float(occ), float(hw["n_cu"]), 0.0, h2, rows_valid, cols_valid,
                            one_tile_row=tiles_m == 1)
        l_sk = stream_k_phase(hw, v, occ, slots, left, per_worker, full["l_compute"], no_l2)
        l_sum = stream_k_sum(hw, v, slots, left)
        for name in ("l_compute", "l_issue", "l_lds", "l_l2", "l_mall", "l_hbm", "l_mem", "l_prologue", "l_epilogue",
                     "l_iter", "l_tile"):
            out[name] = full[name]
        out.update(waves=whole + left / slots, active_cu=hw["n_cu"], l_mem_tail=full["l_mem"], l_tile_tail=l_sk,
                   l_reduce=l_sum, l_total=hw["launch_clk"] + whole * full["l_tile"] + l_sk + l_sum)
    out["total_us"] = out["l_total"] / (hw["clk_ghz"] * 1e3)
    return out


def predict_grouped(hw, dtype, shapes, v, b_layout=0):
    """ONE launch of several products [(M, N, K), ...] (M = 0: an empty group) with variant v, no K
    splitting.  READING (Sections II-B and V-C only name the grouped dimension): Algorithm 4 counts all
    groups' tiles together; Algorithm 8 prices each group's tile on a full device with that group's own
    cache tile, hit rates and K loop; Algorithm 9 is the wave count times the tile-weighted mean of the
    groups' tile latencies, plus one launch.  -> (l_total, [group_m per group])"""
    es = _elem_bytes(dtype)
    counts, latencies, bands = [], [], []
    for (M, N, K) in shapes:
        if M == 0:
            bands.append(1)
            continue
        p = predict(hw, dtype, M, N, K, v, 1, b_layout=b_layout)
        counts.append((-(-M // v["block_m"])) * (-(-N // v["block_n"])))
        latencies.append(p["l_tile_full"])
        bands.append(p["group_m"])
    total_tiles = sum(counts)
    mean_tile = sum(c * l for c, l in zip(counts, latencies)) / total_tiles
    slots = hw["n_cu"] * resident_workgroups(hw, v, es)
    return hw["launch_clk"] + math.ceil(total_tiles / slots) * mean_tile, bands
