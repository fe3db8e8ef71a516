"""Host checks of the Stream-K work split (no GPU): the C ABI exposes the arithmetic the kernel and
the summation pass run, and the properties that make the result a GEMM are checked by brute force:
every K slab of every stream-K tile is computed exactly once, ranges are balanced, and the
summation pass adds up exactly the partials that were written."""
import pytest

from paper_2512_04226_amd import binding as g


def _stream_k_cfgs(M, N, K, dtype=0):
    out = []
    for idx in range(g.gemm_cfg_count(dtype)):
        c = g.gemm_cfg_at(idx, M, N, K, dtype)
        if c is not None and c.stream_k:
            out.append(c)
    return out


def _raster(tiles_m, tiles_n, group_m, t):
    """Tile coordinates of logical id t: column-major inside bands of group_m tile rows."""
    band = t // (group_m * tiles_n)
    first = band * group_m
    rows = min(group_m, tiles_m - first)
    r = t - band * group_m * tiles_n
    return first + r % rows, r // rows


def _check_plan(c):
    G, sk_tiles, dp_tiles, S = g.gemm_stream_k_plan(c)
    tiles_m, tiles_n = -(-c.M // c.block_m), -(-c.N // c.block_n)
    assert G == c.sk_workers and S == -(-c.K // c.block_k)
    assert sk_tiles + dp_tiles == tiles_m * tiles_n and sk_tiles == (tiles_m * tiles_n) % G and 0 < sk_tiles
    cover = [[0] * S for _ in range(sk_tiles)]
    writers = [[] for _ in range(sk_tiles)]      # (worker, segment number, complete) per tile, in worker order
    sizes = []
    for w in range(G):
        segs = g.gemm_stream_k_segments(c, w)
        assert 1 <= len(segs) <= 2
        sizes.append(sum(s.count for s in segs))
        for i, s in enumerate(segs):
            assert 0 <= s.sk_tile < sk_tiles and s.count >= 1 and 0 <= s.slab0 and s.slab0 + s.count <= S
            assert (s.tile_m, s.tile_n) == _raster(tiles_m, tiles_n, c.group_m, dp_tiles + s.sk_tile)
            assert s.complete == int(s.count == S)
            for k in range(s.slab0, s.slab0 + s.count):
                cover[s.sk_tile][k] += 1
            writers[s.sk_tile].append((w, i, s.complete))
        if len(segs) == 2:      # a worker's range is contiguous: end of one tile, start of the next
            assert segs[0].slab0 + segs[0].count == S and segs[1].slab0 == 0 and segs[1].sk_tile == segs[0].sk_tile + 1
    assert all(v == 1 for row in cover for v in row)
    assert max(sizes) - min(sizes) <= 1 and sum(sizes) == sk_tiles * S
    for j in range(sk_tiles):
        first, last, slot = g.gemm_stream_k_contributors(c, j)
        ws = writers[j]
        assert [w for w, _, _ in ws] == list(range(first, last + 1))
        if first == last:
            assert ws[0][2] == 1          # stored by its only worker, nothing to sum
        else:
            assert all(cpl == 0 for _, _, cpl in ws)
            assert ws[0][1] == slot and all(i == 0 for _, i, _ in ws[1:])
    return G, sk_tiles, dp_tiles, S


@pytest.mark.parametrize("shape", [(8448, 8448, 8192), (768, 768, 2048), (1808, 7344, 272), (300, 520, 4096),
                                   (16, 28672, 8192), (4352, 4096, 512)])
def test_every_enumerated_stream_k_cfg_covers_each_slab_once(shape):
    cfgs = _stream_k_cfgs(*shape)
    assert cfgs, "no stream-K candidate for %s" % (shape,)
    for c in cfgs:
        _check_plan(c)
        assert g.gemm_workspace_bytes(c) == 2 * c.sk_workers * c.block_m * c.block_n * 4


def test_hand_set_worker_counts_including_whole_tile_workers():
    base = next(c for c in _stream_k_cfgs(768, 768, 2048) if (c.block_m, c.block_n, c.block_k) == (256, 256, 64))
    seen_two = False
    for G in (2, 4, 5, 7, 8, 10, 17, 33, 64, 100, 255):
        c = base.copy()
        c.sk_workers = G
        tiles = 9
        if tiles % G == 0 or (tiles % G) * 32 < G:
            with pytest.raises(g.GemmError):
                g.gemm_stream_k_plan(c)
            continue
        _check_plan(c)
        for w in range(G):
            segs = g.gemm_stream_k_segments(c, w)
            seen_two |= len(segs) == 2
    assert seen_two
    c = base.copy()
    c.K, c.lda = 64, 64            # S = 1: every range is a whole tile
    c.sk_workers = 5               # 9 % 5 = 4 tiles, 4 iterations < 5 workers: not a plan
    with pytest.raises(g.GemmError):
        g.gemm_stream_k_plan(c)
    c.K, c.lda, c.sk_workers = 128, 128, 5      # S = 2, 4 tiles, 8 iterations over 5 workers:
    _check_plan(c)                              # ranges [0,1) [1,3) [3,4) [4,6) [6,8): two of them are whole tiles
    whole = [w for w in range(5) for s in g.gemm_stream_k_segments(c, w) if s.complete]
    assert whole == [3, 4]


def test_stream_k_errors():
    c = g.gemm_select(512, 512, 512, 0)
    if not c.stream_k:
        with pytest.raises(g.GemmError):
            g.gemm_stream_k_plan(c)
    sk = _stream_k_cfgs(8448, 8448, 8192)[0]
    G = sk.sk_workers
    with pytest.raises(g.GemmError):
        g.gemm_stream_k_segments(sk, G)
    with pytest.raises(g.GemmError):
        g.gemm_stream_k_segments(sk, -1)
    with pytest.raises(g.GemmError):
        g.gemm_stream_k_contributors(sk, g.gemm_stream_k_plan(sk)[1])
    bad = sk.copy(); bad.split_k = 2
    with pytest.raises(g.GemmError):
        g.gemm_stream_k_plan(bad)
    bad = sk.copy(); bad.sk_workers = 0
    with pytest.raises(g.GemmError):
        g.gemm_stream_k_plan(bad)


def test_model_prefers_stream_k_for_a_small_tail_on_a_deep_problem():
    """33 x 33 tiles of 256 x 256 on 256 CUs: four whole waves and 65 tiles left; splitting those
    along K beats a fifth, quarter-full wave (Section II-A's wave-quantisation example)."""
    sk = [c for c in _stream_k_cfgs(8448, 8448, 8192) if (c.block_m, c.block_n, c.block_k, c.waves_n) == (256, 256, 64, 4)][0]
    dp = next(c for c in (g.gemm_cfg_at(i, 8448, 8448, 8192, 0) for i in range(g.gemm_cfg_count(0)))
              if c is not None and c.kernel_id == sk.kernel_id and c.split_k == 1 and not c.stream_k)
    p_sk, p_dp = g.gemm_predict(sk), g.gemm_predict(dp)
    assert p_dp.waves == 5 and p_sk.waves == pytest.approx(4 + 65 / 256)
    assert p_sk.total_us < 0.93 * p_dp.total_us
    # and not when the last wave is nearly full: 16 x 15 = 240 tiles of 256
    nearly = [c for c in _stream_k_cfgs(4096, 3840, 8192) if c.kernel_id == sk.kernel_id]
    if nearly:
        full = next(c for c in (g.gemm_cfg_at(i, 4096, 3840, 8192, 0) for i in range(g.gemm_cfg_count(0)))
                    if c is not None and c.kernel_id == sk.kernel_id and c.split_k == 1 and not c.stream_k)
        assert g.gemm_predict(nearly[0]).total_us > g.gemm_predict(full).total_us
