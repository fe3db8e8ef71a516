"""Device calibration of the model's constants (a one-off, offline step; never run by
gemm_select or gemm_run):

  * L_MI of every matrix instruction and the HBM streaming rate, from the library's probes;
  * SLAB_CLK of every kernel variant: steady-state clocks per K slab of one tile on a full CU,
    from one large compute-bound problem per datatype (8192^3).

Prints the hardware lines and the variants.hpp rows with the two measured columns (B row-major,
B K-contiguous).

    python -m paper_2512_04226_amd.calibrate [--n 8192]
"""
import argparse

import numpy as np
import torch

from . import binding as g
from .sweep import Workspace, make_operands


def measure_rates():
    scratch = torch.zeros(16, dtype=torch.float32, device="cuda")
    hw = g.gemm_hw_get()
    out = {}
    for dt, name in ((g.GEMM_BF16, "bf16"), (g.GEMM_FP8_E4M3, "fp8")):
        for mi in (32, 16):
            tf = g.gemm_probe_mfma(dt, mi, scratch)
            k = {(0, 32): 16, (0, 16): 32, (1, 32): 64, (1, 16): 128}[(dt, mi)]
            flop = 2.0 * mi * mi * k
            l_mi = flop * hw.n_cu * hw.simd_per_cu * hw.clk_ghz / (tf * 1e3)
            out[(name, mi)] = (tf, l_mi)
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)     # 1 GiB > MALL
    out["hbm_gbps"] = g.gemm_probe_stream(buf, scratch)
    return out


def _time_plain(cfg, A, B, C, launches=10):
    """Microseconds per launch: plain back-to-back launches between two events, after two warm-ups
    (how an application, and bench.py, sees the kernel)."""
    for _ in range(2):
        g.gemm_run(cfg, A, B, C)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        g.gemm_run(cfg, A, B, C)
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / launches


def measure_slab_clk(dtype, n, b_layout=0, passes=5):
    """Median over `passes` sweeps of the variant list, each in a different order: the chip is
    power-limited on these shapes, so what ran just before moves a timing by a few percent."""
    hw = g.gemm_hw_get()
    A, B, C = make_operands(n, n, n, dtype, normal=True)     # the headline workload's value distribution
    ws = Workspace()
    cfgs = []
    seen = set()
    for idx in range(g.gemm_cfg_count(dtype)):
        cfg = g.gemm_cfg_at_ex(idx, n, n, n, dtype, b_layout)
        if cfg is None or cfg.split_k != 1 or cfg.stream_k or cfg.kernel_id in seen:
            continue
        seen.add(cfg.kernel_id)
        ws.ensure(cfg)
        cfgs.append(cfg)
    times = {c.kernel_id: [] for c in cfgs}
    rng = np.random.default_rng(0)
    for p in range(passes):
        order = list(range(len(cfgs)))
        if p % 2:
            order.reverse()
        if p >= 2:
            rng.shuffle(order)
        for i in order:
            times[cfgs[i].kernel_id].append(_time_plain(cfgs[i], A, B, C))
    rows = []
    for cfg in cfgs:
        us = float(np.median(times[cfg.kernel_id]))
        tiles = -(-n // cfg.block_m) * -(-n // cfg.block_n)
        slabs = -(-n // cfg.block_k)
        clk = us * hw.clk_ghz * 1e3 - hw.launch_clk
        rows.append((cfg, us, clk * hw.n_cu / (tiles * slabs)))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=8192)
    ap.add_argument("--skip-rates", action="store_true")
    args = ap.parse_args()
    if not args.skip_rates:
        r = measure_rates()
        for key, val in r.items():
            if key == "hbm_gbps":
                print("HBM streaming read: %.0f GB/s" % val)
            else:
                print("MFMA %s %dx%d: %.0f TFLOP/s device-wide -> L_MI = %.1f clk" % (key[0], key[1], key[1], val[0], val[1]))
    for dtype, name in ((g.GEMM_BF16, "BF16"), (g.GEMM_FP8_E4M3, "FP8")):
        print("// %s variants, SLAB_CLK measured on %d^3" % (name, args.n))
        rows = measure_slab_clk(dtype, args.n, 0)
        rows_kc = measure_slab_clk(dtype, args.n, 1)
        for (cfg, us, tau), (_, us_kc, tau_kc) in zip(rows, rows_kc):
            # the K-contiguous gain of a small tile on this huge problem (L2-resident panels, hundreds of
            # waves) is larger than what the small problems that pick such tiles see: floor it
            tau_kc = max(tau_kc, 0.9 * tau)
            print("    X(%d, %d, %d, %d, %d, %d, %d, %d, %d)   // %.1f us %.0f TFLOP/s | K-contiguous B %.1f us %.0f TFLOP/s" % (
                cfg.block_m, cfg.block_n, cfg.block_k, cfg.waves_m, cfg.waves_n, cfg.mfma, cfg.stages, round(tau),
                round(tau_kc), us, 2.0 * args.n ** 3 / us * 1e-6, us_kc, 2.0 * args.n ** 3 / us_kc * 1e-6), flush=True)


if __name__ == "__main__":
    main()
