"""Plain transcription of the paper's analytical model (TEST INFRASTRUCTURE ONLY).

Section IV of the paper: Algorithm 3 (compute latency of a shared-memory tile), Algorithm 4
(active CUs in the last timestep, number of waves), Algorithm 5 (cache hit rate of a cache
tile), Algorithm 6 (factorisations of the CU count of a cache scope), Algorithm 7 (memory
latency of one loop iteration), Algorithm 8 (latency of one output tile) and Algorithm 9
(total latency).  The `alg*` functions take the steps in the paper's order and notation,
with no reading added.  `predict` composes them for one kernel variant the way the shipped
selector is specified to (every place where the paper is silent or inconsistent is marked
READING); the tests compare the C++ selector's terms with it.

Shares no code with the product; nothing under the product package imports this module.
The selector's final pick is a heuristic ranked empirically against a sweep, so beyond the
structural pins in tests/test_selector_model.py its parity is unpinned by the paper.
"""
import math


# ---------------------------------------------------------------- the paper's algorithms

def alg3_compute_latency(mi_m, mi_n, mi_k, mt_m, mt_n, mt_k, l_mi):
    """Algorithm 3: matrix instructions per shared-memory tile and their latency."""
    n_mi_m = math.ceil(mt_m / mi_m)
    n_mi_n = math.ceil(mt_n / mi_n)
    n_mi_k = math.ceil(mt_k / mi_k)
    n_mi = n_mi_m * n_mi_n * n_mi_k
    l_mt = l_mi * n_mi
    return n_mi, l_mt


def alg4_occupancy(M, N, mt_m, mt_n, n_cu):
    """Algorithm 4 as printed: (active_cu, omega, T_out); active_cu is T_out mod N_CU."""
    n_mt_m = math.ceil(M / mt_m)
    n_mt_n = math.ceil(N / mt_n)
    t_out = n_mt_m * n_mt_n
    omega = math.ceil(t_out / n_cu)
    active_cu = t_out % n_cu
    return active_cu, omega, t_out


def alg5_hit_rate(m_t, n_t, M_T, N_T, K_T):
    """Algorithm 5: hit rate of an m_t x n_t cache tile of M_T x N_T x K_T workgroup tiles."""
    U = (m_t * M_T + n_t * N_T) * K_T          # uncached reads
    R = (m_t * n_t) * (M_T + N_T) * K_T        # total reads
    h = 1 - U / R
    return h


def alg6_factorizations(n_cu_cache):
    """Algorithm 6: every (f_m, f_n) with f_m * f_n = N_CU_cache, in ascending f_m."""
    F = []
    for i in range(1, n_cu_cache + 1):
        if n_cu_cache % i == 0:
            F.append((i, n_cu_cache // i))
    return F


def alg7_memory_latency(ld_cu, C, H1, H2, R_L1, R_1, R_2, R_MEM, L_lat):
    """Algorithm 7 as printed (any consistent unit of data per cycle)."""
    L_cu_lat = ld_cu / R_L1
    T = ld_cu * C
    L_1 = T / R_1
    T_2 = (1 - H1) * T
    L_2 = T_2 / R_2
    T_M = (1 - H2) * T_2
    L_MEM = T_M / R_MEM + L_lat
    return max(L_cu_lat, L_1, L_2, L_MEM)


def alg8_tile_latency(K, k_t, l_mem, l_compute, a, m_t, n_t, R_mem):
    """Algorithm 8 as printed."""
    l_prologue = l_mem
    l_epilogue = a * m_t * n_t / R_mem
    l_loopiter = max(l_compute, l_mem)
    I = math.ceil(K / k_t) - 1
    return l_prologue + l_epilogue + l_loopiter * I


def alg9_total_latency(M, N, m_t, n_t, n_cu, l_tile):
    """Algorithm 9 as printed."""
    n_m = math.ceil(M / m_t)
    n_n = math.ceil(N / n_t)
    n_waves = math.ceil(n_m * n_n / n_cu)
    return n_waves * l_tile


# ---------------------------------------------------------------- composition with readings

def _ceil_div(a, b):
    return -(-a // b)


def occupancy(hw, v, es):
    """READING: workgroups of variant v resident on one CU (LDS ring, register estimate, 8 at most)."""
    lds = v["stages"] * (v["block_m"] + v["block_n"]) * v["block_k"] * es
    waves = v["waves_m"] * v["waves_n"]
    acc = v["block_m"] * v["block_n"] / (waves * 64.0)      # fp32 accumulators per lane
    vgpr = acc + 64.0
    waves_per_simd = max(1, min(8, int(512.0 // vgpr)))
    by_regs = max(1, waves_per_simd * hw["simd_per_cu"] // waves)
    by_lds = max(1, int(hw["lds_bytes"] // lds))
    return max(1, min(by_regs, by_lds, 8))


def choose_cache_tile(scope, v, tiles_m, tiles_n):
    """READING: among Algorithm 6's pairs, clipped to the tile grid, the one with the highest
    Algorithm-5 hit rate; ties -> cache tile closest to square in elements -> wider."""
    best = None
    for (i, j) in alg6_factorizations(scope):
        fm, fn = min(i, tiles_m), min(j, tiles_n)
        h = min(1.0, max(0.0, alg5_hit_rate(fm, fn, v["block_m"], v["block_n"], v["block_k"])))
        skew = abs(fm * v["block_m"] - fn * v["block_n"])
        better = False
        if best is None or h > best["h"] + 1e-12:
            better = True
        elif abs(h - best["h"]) <= 1e-12:
            if skew < best["skew"] - 1e-9:
                better = True
            elif abs(skew - best["skew"]) <= 1e-9 and fn > best["fn"]:
                better = True
        if better:
            best = {"h": h, "skew": skew, "fm": fm, "fn": fn, "raw": i}
    return best


def segment_efficiency(hw, seg):
    """READING: share of the HBM rate reached with `seg` contiguous bytes per matrix row."""
    if seg >= 256:
        return 1.0
    s = max(seg, 32.0)
    return min(1.0, hw["seg_eff_lo"] + (1.0 - hw["seg_eff_lo"]) * math.log2(s / 32.0) / 3.0)


def stream_k_split(tiles, slots, slabs):
    """Hybrid Stream-K split (Section V-E names Stream-K as the paper kernels' answer to wave
    quantisation; READING: whole waves of `slots` tiles stay one-tile-per-workgroup, the
    tiles % slots left over are cut along K into `slots` equal ranges).  Returns (whole waves,
    stream-K tiles, slabs per worker) or None when there is no partial wave or fewer slabs than
    workers."""
    sk = tiles % slots
    if sk == 0 or sk * slabs < slots:
        return None
    return (tiles - sk) // slots, sk, sk * slabs / slots


def predict(hw, dtype, M, N, K, v, split_k, b_layout=0, stream_k=0, batch=1):
    """Model terms for variant v (dict: block_m/n/k, waves_m/n, mfma, stages, slab_clk) with the
    reduction split split_k ways; hw is a dict of the hardware descriptor's fields; b_layout 0 =
    B row-major K x N, 1 = B stored K-contiguous (then v["slab_clk"] is that layout's constant);
    stream_k = 1 prices the hybrid Stream-K split of the last partial wave (needs split_k = 1);
    batch = number of independent problems of this shape in one launch (READING: Section II-B only
    names the batch dimension; here it multiplies the tile count of Algorithm 4 and the reduction
    pass's bytes).
    Returns a dict with the names of the C ABI's gemm_prediction plus group_m."""
    # dtype 0 bf16, 1 fp8 e4m3, 2 fp16.  READING: fp16 shares bf16's instruction shapes and rates.
    row = 1 if dtype == 1 else 0
    es = 1 if dtype == 1 else 2
    mi = v["mfma"]
    mi_k = {(0, 32): 16, (0, 16): 32, (1, 32): 64, (1, 16): 128}[(row, mi)]
    waves_wg = v["waves_m"] * v["waves_n"]
    out = {}

    # Algorithm 3 (count, and latency at full utilisation spread over the workgroup's SIMDs)
    l_mi = hw["l_mi_clk"][row][0 if mi == 32 else 1]
    n_mi, l_mt = alg3_compute_latency(mi, mi, mi_k, v["block_m"], v["block_n"], v["block_k"], l_mi)
    out["n_mi"] = n_mi
    out["l_mt_ideal"] = l_mt / min(hw["simd_per_cu"], waves_wg)

    # Algorithm 4.  READING: K slices count as tiles, a CU offers `occ` slots, a remainder of 0
    # means a full last wave.
    _, _, t_out = alg4_occupancy(M, N, v["block_m"], v["block_n"], hw["n_cu"])
    tiles_m, tiles_n = _ceil_div(M, v["block_m"]), _ceil_div(N, v["block_n"])
    tiles = t_out * split_k * batch
    occ = occupancy(hw, v, es)
    slots = hw["n_cu"] * occ
    waves = math.ceil(tiles / slots)
    tail_tiles = tiles - (waves - 1) * slots
    active = min(tail_tiles, hw["n_cu"])
    tail_per_cu = math.ceil(tail_tiles / hw["n_cu"])
    out.update(tiles=tiles, waves=waves, active_cu=active)

    # Algorithms 5/6 + capacity derate (READING: h * min(1, eff * capacity / footprint))
    l2_scope = hw["n_cu"] // hw["n_xcd"] * occ
    c1 = choose_cache_tile(l2_scope, v, tiles_m, tiles_n)
    c2 = choose_cache_tile(hw["n_cu"] * occ, v, tiles_m, tiles_n)
    # READING: rows and columns of a tile that lie outside the matrix are never fetched, so the
    # bytes a tile loads and Algorithm 5's unique / requested counts use the mean valid extent of
    # a tile, M / tiles_m by N / tiles_n, instead of the nominal M_T by N_T.
    bm_e, bn_e = M / tiles_m, N / tiles_n
    for c in (c1, c2):
        c["h"] = min(1.0, max(0.0, alg5_hit_rate(c["fm"], c["fn"], bm_e, bn_e, v["block_k"])))
    fp1 = (c1["fm"] * v["block_m"] + c1["fn"] * v["block_n"]) * v["block_k"] * es * 2.0
    fp2 = (c2["fm"] * v["block_m"] + c2["fn"] * v["block_n"]) * v["block_k"] * es * 2.0
    h1 = c1["h"] * min(1.0, hw["cache_eff_frac"] * hw["l2_bytes"] / fp1)
    h2 = c2["h"] * min(1.0, hw["cache_eff_frac"] * hw["mall_bytes"] / fp2)
    out.update(f_m=c1["fm"], f_n=c1["fn"], h_l2=h1, h_mall=h2)
    out["group_m"] = max(1, min(c1["raw"], tiles_m))

    k_slabs = _ceil_div(K, v["block_k"])
    slabs = _ceil_div(k_slabs, split_k)              # slabs per K slice
    out["iters"] = slabs - 1
    out_bytes = 4.0 if split_k > 1 else 2.0

    def memory(per_cu, act, h_l2=None, per_cu_mem=None):
        # Algorithm 7 in bytes and clocks.  READING: Ld_CU = (BM + BN) * BK bytes per tile; an LDS
        # fragment-read term is added; the HBM term carries the row-segment efficiency and the
        # latency is shared by the slabs in flight.
        hit1 = h1 if h_l2 is None else h_l2
        # every load instruction of the nominal tile is issued; only the valid extent moves bytes
        l_issue = (v["block_m"] + v["block_n"]) * v["block_k"] * es * per_cu / hw["vmem_bytes_per_clk"]
        pcm = per_cu if per_cu_mem is None else per_cu_mem
        a_bytes = bm_e * v["block_k"] * es * pcm
        b_bytes = bn_e * v["block_k"] * es * pcm
        ld_cu = a_bytes + b_bytes
        # READING: K-contiguous B is read with ds_read_b128 like A, row-major B with transpose reads
        b_rate = hw["lds_bytes_per_clk"] if b_layout else hw["lds_tr_bytes_per_clk"]
        l_lds = (v["block_m"] * v["waves_n"] * v["block_k"] * es / hw["lds_bytes_per_clk"]
                 + v["block_n"] * v["waves_m"] * v["block_k"] * es / b_rate) * per_cu
        total = ld_cu * act
        xcds = min(hw["n_xcd"], max(1.0, act))
        l_l2 = (total / xcds) / hw["l2_bytes_per_clk"]
        l_mall = (1.0 - hit1) * total / hw["mall_bytes_per_clk"]
        ea = segment_efficiency(hw, v["block_k"] * es)
        eb = segment_efficiency(hw, (v["block_k"] if b_layout else v["block_n"]) * es)
        # READING: Algorithm 7 multiplies (1 - H1)(1 - H2), but both rates come from Algorithm 5 on
        # nested scopes, so H2 already contains the reuse H1 counts; the product would let fewer
        # bytes reach HBM than the matrices hold.  The share of requested bytes that reaches HBM is
        # what neither scope can serve: min(1 - H1, 1 - H2).
        t_m = min(1.0 - h2, 1.0 - hit1) * (a_bytes / ea + b_bytes / eb) * act
        l_hbm = t_m / hw["hbm_bytes_per_clk"] + hw["mem_latency_clk"] / max(1.0, per_cu * (v["stages"] - 1))
        return dict(l_issue=l_issue, l_lds=l_lds, l_l2=l_l2, l_mall=l_mall, l_hbm=l_hbm,
                    l_mem=max(l_issue, l_lds, l_l2, l_mall, l_hbm))

    def tile(per_cu, act, per_cu_mem=None):
        # READING of Algorithm 3's "high utilisation" assumption: the compute latency of a slab is
        # the variant's measured slab cost, scaled when the CU holds fewer tiles than fit.
        l_comp = v["slab_clk"] * per_cu
        if per_cu < occ:
            l_comp *= hw["under_occ_frac"] + (1.0 - hw["under_occ_frac"]) * per_cu / occ
        m = memory(per_cu, act, per_cu_mem=per_cu_mem)
        # Algorithm 8.  READING: fixed latency and per-workgroup cost in the prologue, output bytes
        # through the HBM rate plus a fixed cost in the epilogue, one exposed compute drain.
        l_pro = m["l_mem"] + hw["mem_latency_clk"] + hw["wg_overhead_clk"]
        l_epi = act * per_cu * v["block_m"] * v["block_n"] * out_bytes / hw["hbm_bytes_per_clk"] + hw["epilogue_clk"]
        l_iter = max(l_comp, m["l_mem"])
        l_tile = l_pro + l_epi + l_iter * (slabs - 1) + l_comp
        return dict(m, l_compute=l_comp, l_prologue=l_pro, l_epilogue=l_epi, l_iter=l_iter, l_tile=l_tile)

    full = tile(float(occ), float(hw["n_cu"]))
    # READING: in the last wave a CU computes ceil(tail / active) tiles, but the bytes that wave moves
    # are those of the tiles that exist: tail / active per CU.
    tail = tile(float(tail_per_cu), float(active), tail_tiles / active)
    shown = full if waves > 1 else tail
    for k in ("l_compute", "l_issue", "l_lds", "l_l2", "l_mall", "l_hbm", "l_mem", "l_prologue", "l_epilogue",
              "l_iter", "l_tile"):
        out[k] = shown[k]
    out["l_mem_tail"] = tail["l_mem"]
    out["l_tile_tail"] = tail["l_tile"]
    out["l_tile_full"] = full["l_tile"]      # Algorithm 8 on a full device, whatever this problem's own wave count

    l_reduce = 0.0
    if split_k > 1:
        nbytes = M * N * (4.0 * split_k + 2.0) * batch
        rate = hw["mall_bytes_per_clk"] if nbytes <= hw["cache_eff_frac"] * hw["mall_bytes"] else hw["hbm_bytes_per_clk"]
        l_reduce = hw["reduce_launch_clk"] + nbytes / rate
    out["l_reduce"] = l_reduce
    # Algorithm 9.  READING: full waves and the under-occupied last wave are priced separately,
    # plus one launch; with two or more workgroups resident per CU a share overlap_frac of a tile's
    # prologue and store stage hides under the other workgroups' K loops in every wave that is
    # followed by another.
    hidden = hw["overlap_frac"] * (full["l_prologue"] + full["l_epilogue"]) if (occ >= 2 and waves > 1) else 0.0
    out["l_total"] = hw["launch_clk"] + (waves - 1) * (full["l_tile"] - hidden) + tail["l_tile"] + l_reduce

    if stream_k:
        # READING (fractional waves in Algorithms 4 and 9): after `whole` full waves the remaining
        # sk tiles cost w slabs per slot instead of a whole tile; every CU is full; a share
        # sk/slots of the workers works on two tiles and pays prologue and store stage twice;
        # partial tiles are fp32 and a second pass reads (slots + sk) of them and writes sk tiles.
        whole, sk, w = stream_k_split(tiles, slots, slabs)
        tile_elems = v["block_m"] * v["block_n"]
        # READING: workers that share an L2 sit at different K offsets of different tiles, so the
        # stream-K phase is priced with an L2 hit rate of zero.
        m_sk = memory(float(occ), float(hw["n_cu"]), h_l2=0.0)
        iter_sk = max(full["l_compute"], m_sk["l_mem"])
        pro_sk = m_sk["l_mem"] + hw["mem_latency_clk"] + hw["wg_overhead_clk"]
        l_epi_sk = hw["n_cu"] * occ * tile_elems * 4.0 / hw["hbm_bytes_per_clk"] + hw["epilogue_clk"]
        l_sk = (1.0 + sk / slots) * (pro_sk + l_epi_sk) + iter_sk * (w - 1.0) + full["l_compute"]
        nbytes = (slots + sk) * tile_elems * 4.0 + sk * tile_elems * 2.0
        rate = hw["mall_bytes_per_clk"] if nbytes <= hw["cache_eff_frac"] * hw["mall_bytes"] else hw["hbm_bytes_per_clk"]
        # READING: one output's contributors (at most slots // sk + 2) are added by 1, 4 or 8 thread
        # rows, chosen by that count, with 4 loads in flight each
        contrib = slots // sk + 2
        rows = 8 if contrib > 32 else 4 if contrib > 8 else 1
        chain = math.ceil(contrib / (4.0 * rows)) * hw["mem_latency_clk"]
        l_sum = hw["reduce_launch_clk"] + nbytes / rate + chain
        for k in ("l_compute", "l_issue", "l_lds", "l_l2", "l_mall", "l_hbm", "l_mem", "l_prologue", "l_epilogue",
                  "l_iter", "l_tile"):
            out[k] = full[k]
        out.update(waves=whole + sk / slots, active_cu=hw["n_cu"], l_mem_tail=full["l_mem"], l_tile_tail=l_sk,
                   l_reduce=l_sum, l_total=hw["launch_clk"] + whole * full["l_tile"] + l_sk + l_sum)
    out["total_us"] = out["l_total"] / (hw["clk_ghz"] * 1e3)
    return out


def predict_grouped(hw, dtype, shapes, v, b_layout=0):
    """Total latency in clocks of ONE launch that computes several products of different shapes
    [(M, N, K), ...] (M = 0: an empty group) with variant v, no K splitting.
    READING (Sections II-B and V-C only name the grouped dimension): Algorithm 4 counts the tiles
    of all groups together, T = sum T_g, omega = ceil(T / slots); Algorithm 8 prices each group's
    tile on a full device (the other groups' tiles keep the CUs busy) with that group's own cache
    tile, hit rates and K loop; Algorithm 9 becomes omega times the tile-weighted mean of the
    groups' tile latencies, plus one launch.  Returns (l_total, [group_m per group])."""
    es = 1 if dtype == 1 else 2
    tiles, weighted, group_m = 0, 0.0, []
    for (M, N, K) in shapes:
        if M == 0:
            group_m.append(1)
            continue
        p = predict(hw, dtype, M, N, K, v, 1, b_layout=b_layout)
        t = _ceil_div(M, v["block_m"]) * _ceil_div(N, v["block_n"])
        tiles += t
        weighted += t * p["l_tile_full"]
        group_m.append(p["group_m"])
    slots = hw["n_cu"] * occupancy(hw, v, es)
    return hw["launch_clk"] + math.ceil(tiles / slots) * weighted / tiles, group_m
