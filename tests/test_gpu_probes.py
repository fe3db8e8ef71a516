"""The calibration probes (Section I of the paper: the model's rates come from micro-benchmarks) on the
device: every probe returns a finite rate inside the window its published peak allows, and repeats."""
import math

import pytest
import torch

pytestmark = pytest.mark.gpu

PEAK_TFLOPS = {0: 2500.0, 1: 5000.0}
# the published peaks are quoted at 2.4 GHz; a cool chip holds a little more on the short constant-operand loop
# (5006 TFLOP/s fp8 was measured), so the upper bounds allow 3 %
ABOVE = 1.03
PEAK_HBM_GBPS = 8000.0


@pytest.fixture(scope="module")
def g():
    from paper_2512_04226_amd import binding
    return binding


@pytest.fixture(scope="module")
def scratch():
    return torch.zeros(16, dtype=torch.float32, device="cuda")


@pytest.mark.parametrize("dtype,mfma", [(0, 32), (1, 32)])
def test_mfma_probe_is_within_the_published_peak_and_repeats(g, scratch, dtype, mfma):
    a = g.gemm_probe_mfma(dtype, mfma, scratch)
    b = g.gemm_probe_mfma(dtype, mfma, scratch)
    for x in (a, b):
        assert math.isfinite(x) and 0.5 * PEAK_TFLOPS[dtype] <= x <= ABOVE * PEAK_TFLOPS[dtype], (a, b)
    assert abs(a - b) <= 0.10 * max(a, b), (a, b)


def test_stream_probe_is_within_the_published_peak_and_repeats(g, scratch):
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    a = g.gemm_probe_stream(buf, scratch)
    b = g.gemm_probe_stream(buf, scratch)
    for x in (a, b):
        assert math.isfinite(x) and 0.5 * PEAK_HBM_GBPS <= x <= 1.0 * PEAK_HBM_GBPS, (a, b)
    assert abs(a - b) <= 0.10 * max(a, b), (a, b)


@pytest.mark.parametrize("dtype,mfma", [(0, 32), (0, 16), (1, 32), (1, 16)])
def test_mfma_probe_on_workload_like_operands(g, scratch, dtype, mfma):
    """The settled ceiling on N(0,1)-like register contents: finite, below the published peak, not above
    what the same loop reaches on constant operands (plus timing noise)."""
    const = g.gemm_probe_mfma_ex(dtype, mfma, 0, scratch, warm_ms=20.0, timed_ms=10.0)
    rnd = g.gemm_probe_mfma_ex(dtype, mfma, 1, scratch, warm_ms=20.0, timed_ms=10.0)
    print("mfma_ex dtype %d %dx%d: constant %.0f, workload-like %.0f TFLOP/s" % (dtype, mfma, mfma, const, rnd))
    for x in (const, rnd):
        assert math.isfinite(x) and 0.2 * PEAK_TFLOPS[dtype] <= x <= ABOVE * PEAK_TFLOPS[dtype], (const, rnd)
    assert rnd <= 1.05 * const, (const, rnd)


def test_read_probe_orders_the_memory_levels(g, scratch):
    """Repeated reads of 16 MiB (L2-resident), 128 MiB (MALL-resident) and 1 GiB (HBM): each level is at
    least as fast as the one below it, and the HBM figure agrees with the streaming probe."""
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    l2 = g.gemm_probe_read(buf[:16 << 20], 64, scratch)
    mall = g.gemm_probe_read(buf[:128 << 20], 8, scratch)
    hbm = g.gemm_probe_read(buf, 2, scratch)
    stream = g.gemm_probe_stream(buf, scratch)
    print("read probe: L2 %.0f, MALL %.0f, HBM %.0f GB/s (stream %.0f)" % (l2, mall, hbm, stream))
    assert all(math.isfinite(x) and x > 0 for x in (l2, mall, hbm))
    assert l2 >= 0.95 * mall and mall >= 0.95 * hbm
    assert 0.5 * PEAK_HBM_GBPS <= hbm <= 1.0 * PEAK_HBM_GBPS
    assert abs(hbm - stream) <= 0.15 * stream


def test_lds_probe_rates(g, scratch):
    """A CU's LDS serves at most 256 bytes per clock; transpose reads are not faster than plain ones."""
    hw = g.gemm_hw_get()
    cap = 256.0 * hw.n_cu * 2.6          # GB/s at a generous clock
    rates = {}
    for kind in range(4):
        rates[kind] = max(g.gemm_probe_lds(kind, w, scratch) for w in (4, 8, 16))
        assert math.isfinite(rates[kind]) and 0.1 * cap <= rates[kind] <= cap, rates
    print("lds probe GB/s: b128 %.0f, b64 %.0f, tr_b16 %.0f, tr_b8 %.0f" % tuple(rates[k] for k in range(4)))
    assert rates[2] <= 1.05 * rates[0] and rates[3] <= 1.05 * rates[0]


def test_latency_probe_orders_the_memory_levels(g, scratch):
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    l2 = g.gemm_probe_latency(buf[:2 << 20], scratch)
    hbm = g.gemm_probe_latency(buf, scratch)
    print("latency probe: L2 %.0f ns, HBM %.0f ns" % (l2, hbm))
    assert math.isfinite(l2) and math.isfinite(hbm) and 50.0 <= l2 <= hbm <= 5000.0


def test_fill_probe_orders_the_memory_levels_and_paths(g, scratch):
    """Slabs moved towards LDS by 8-wave workgroups: from L2-resident rows every path runs near the 64 bytes
    per clock a CU's vector memory path delivers, HBM-resident rows arrive at the streaming rate, and writing
    LDS directly is not slower than going through registers and ds_write."""
    hw = g.gemm_hw_get()
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    cap = 64.0 * hw.n_cu * 2.6            # GB/s at a generous clock
    l2 = {k: g.gemm_probe_fill(k, 1, buf, 2048, scratch, sync=1) for k in (0, 1, 2, 3)}
    hbm = {k: g.gemm_probe_fill(k, 2, buf, 1 << 30, scratch, sync=1) for k in (0, 2, 3)}
    wide = g.gemm_probe_fill(0, 3, buf, 1 << 30, scratch)
    stream = g.gemm_probe_stream(buf, scratch)
    print("fill probe GB/s: L2 %s, HBM %s (512-byte pieces %.0f, stream %.0f)" % (
        {k: round(v) for k, v in l2.items()}, {k: round(v) for k, v in hbm.items()}, wide, stream))
    for v in list(l2.values()) + list(hbm.values()) + [wide]:
        assert math.isfinite(v) and v > 0
    for k in l2:
        assert 0.4 * cap <= l2[k] <= cap, l2
    for k in hbm:
        assert 0.5 * PEAK_HBM_GBPS <= hbm[k] <= 1.0 * PEAK_HBM_GBPS and hbm[k] <= l2[k], (hbm, l2)
    assert l2[0] >= 0.8 * l2[3]
    assert abs(hbm[0] - stream) <= 0.25 * stream


def test_probe_argument_checks(g, scratch):
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(g.GemmError):
        g.gemm_probe_mfma_ex(0, 8, 1, scratch)
    with pytest.raises(g.GemmError):
        g.gemm_probe_mfma_ex(5, 32, 1, scratch)
    with pytest.raises(g.GemmError):
        g.gemm_probe_read(small, 4, scratch)
    with pytest.raises(g.GemmError):
        g.gemm_probe_lds(9, 8, scratch)
    with pytest.raises(g.GemmError):
        g.gemm_probe_latency(small, scratch)
    big = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    for bad in ((4, 0, 1 << 20), (0, 4, 1 << 20), (1, 2, 8 << 20), (0, 0, 3 << 20), (0, 0, 32 << 20), (0, 1, 64),
                (0, 2, 1 << 20)):
        with pytest.raises(g.GemmError):
            g.gemm_probe_fill(bad[0], bad[1], big, bad[2], scratch)
    with pytest.raises(g.GemmError):
        g.gemm_probe_fill(0, 1, small, 2048, scratch)
