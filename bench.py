"""Benchmark of the GEMM hot path on one MI355X.

One step = one pass of the whole path over the square bf16 workload: for M=N=K=4096 and
M=N=K=8192 (N(0,1) inputs from seed 1, fp32 accumulate, bf16 output), gemm_select (the
analytical model, host) followed by gemm_run (rasterisation, prologue, K loop, epilogue
on the GPU).  Inputs are resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}   # MI355X dense MFMA, published
PEAK_HBM_GBPS = 8000.0


def ms_per_step_of(tflops, flops_step):
    return flops_step / (tflops * 1e12) * 1e3


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel from the committed counter summary
    (profiles/<name>: a line `traffic_bytes_per_launch: <number>`), or None."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(A, B, rows):
    """The CPU oracle as it stands, timed on a row sample of the 8192^3 workload."""
    import numpy as np
    from oracle import gemm_oracle as oracle

    K, N = B.shape
    sel = np.linspace(0, A.shape[0] - 1, rows).astype(np.int64)
    t0 = time.perf_counter()
    oracle.gemm_rows(A, B, sel, oracle.BF16)
    dt = time.perf_counter() - t0
    flops = 2.0 * rows * N * K
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "%d evenly spaced rows of the 8192^3 product (%.1f s)" % (rows, dt)}


def settled_us(torch, fn, reps=10):
    """Microseconds per call of an enqueueing function in the chip's settled state: at least 30 ms of untimed
    calls first (after idling the chip boosts, then throttles for 15-20 ms before it settles under its power
    limit), then at least `reps` calls and 20 ms timed."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()                               # the first call of a kernel also loads its code
    e0.record()
    for _ in range(2):
        fn()
    e1.record()
    e1.synchronize()
    est_ms = max(e0.elapsed_time(e1) / 2, 1e-3)
    for _ in range(int(30.0 / est_ms) + 1):
        fn()
    reps = max(reps, int(20.0 / est_ms) + 1)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def secondary(also, g, wl, np, torch, dev, sizes, timed_us, ensure_ws):
    """Figures outside the timed region: per-shape rates, the other layouts, precisions and the
    bandwidth-bound path, and the measured ceilings the rooflines are also quoted against."""
    for n in sizes:
        us = timed_us(g.gemm_select(n, n, n, g.GEMM_BF16), *dev[n])
        also["bf16_%d_tflops" % n] = 2.0 * n ** 3 / us * 1e-6
    # the paper's own operand layout (both operands K-contiguous, Section V): same product, B stored N x K
    # cold-cache figure for the size whose operands fit the 256 MB MALL: rotate through four operand
    # sets (4 x 100 MB), so that no launch finds its inputs cached by the previous one
    n_small = sizes[0]
    cfg_s = g.gemm_select(n_small, n_small, n_small, g.GEMM_BF16)
    sets = [dev[n_small]] + [tuple(t.clone() for t in dev[n_small]) for _ in range(3)]
    us_rot = settled_us(torch, lambda: [g.gemm_run(cfg_s, dA, dB, dC) for dA, dB, dC in sets])
    also["bf16_%d_rotating_buffers_tflops" % n_small] = 2.0 * n_small ** 3 * len(sets) / us_rot * 1e-6
    del sets
    n_big = sizes[-1]
    dBt = dev[n_big][1].t().contiguous()
    cfg_kc = g.gemm_select_ex(n_big, n_big, n_big, g.GEMM_BF16, g.GEMM_B_K_CONTIGUOUS)
    us = timed_us(cfg_kc, dev[n_big][0], dBt, dev[n_big][2])
    also["bf16_%d_b_k_contiguous" % n_big] = {"tflops": 2.0 * n_big ** 3 / us * 1e-6, "picked": cfg_kc.describe()}
    del dBt
    # the paper's own precision and layout (Section V): fp16 in / fp16 out, both operands K-contiguous
    Ah, Bh = wl.normal_fp16(n_big, n_big, n_big, seed=1)
    dAh = torch.from_numpy(Ah.view(np.int16)).cuda()
    dBh = torch.from_numpy(np.ascontiguousarray(Bh.T).view(np.int16)).cuda()
    cfg_h = g.gemm_select_ex(n_big, n_big, n_big, g.GEMM_FP16, g.GEMM_B_K_CONTIGUOUS)
    us = timed_us(cfg_h, dAh, dBh, dev[n_big][2])
    also["fp16_%d_b_k_contiguous" % n_big] = {"tflops": 2.0 * n_big ** 3 / us * 1e-6, "picked": cfg_h.describe()}
    del Ah, Bh, dAh, dBh
    scratch = torch.zeros(16, dtype=torch.float32, device="cuda")
    # the matrix cores alone, settled (30 ms untimed, 20 ms timed): on constant operands and on per-lane different
    # N(0,1)-like operands, for both bf16 instruction shapes -- the second is the ceiling the power limit leaves
    # the benchmark's data
    also["mfma_only_bf16_tflops"] = g.gemm_probe_mfma_ex(g.GEMM_BF16, 32, 0, scratch)
    also["mfma_only_bf16_random_tflops"] = {"32x32x16": g.gemm_probe_mfma_ex(g.GEMM_BF16, 32, 1, scratch),
                                            "16x16x32": g.gemm_probe_mfma_ex(g.GEMM_BF16, 16, 1, scratch)}
    also["mfma_only_fp8_random_tflops"] = {"32x32x64": g.gemm_probe_mfma_ex(g.GEMM_FP8_E4M3, 32, 1, scratch),
                                           "16x16x128": g.gemm_probe_mfma_ex(g.GEMM_FP8_E4M3, 16, 1, scratch)}
    n8 = 8192
    Aq, Bq, sa, sb = wl.config4(n8)
    cfg8 = g.gemm_select(n8, n8, n8, g.GEMM_FP8_E4M3)
    cfg8.alpha = float(sa) * float(sb)
    us = timed_us(cfg8, torch.from_numpy(Aq).cuda(), torch.from_numpy(Bq).cuda(), dev[n8][2])
    also["fp8_8192"] = {"tflops": 2.0 * n8 ** 3 / us * 1e-6, "frac_of_fp8_peak": 2.0 * n8 ** 3 / us * 1e-6 / PEAK_TFLOPS["fp8"],
                        "frac_of_measured_ceiling": 2.0 * n8 ** 3 / us * 1e-6 / also["mfma_only_fp8_random_tflops"][
                            "32x32x64" if cfg8.mfma == 32 else "16x16x128"],
                        "picked": cfg8.describe()}
    del Aq, Bq
    Ms, Ns, Ks = 16, 28672, 8192
    As, Bs = wl.config3(Ms, Ns, Ks)
    cfgs = g.gemm_select(Ms, Ns, Ks, g.GEMM_BF16)
    dBs = torch.from_numpy(Bs.view(np.int16)).cuda()
    us = timed_us(cfgs, torch.from_numpy(As.view(np.int16)).cuda(), dBs,
                  torch.empty((Ms, Ns), dtype=torch.int16, device="cuda"))
    sk_bytes = (Ms * Ks + Ks * Ns + Ms * Ns) * 2.0
    also["skinny_bf16_M16_N28672_K8192"] = {"us": us, "gbps": sk_bytes / us * 1e-3,
                                            "frac_of_hbm_peak": sk_bytes / us * 1e-3 / PEAK_HBM_GBPS,
                                            "picked": cfgs.describe()}
    also["hbm_stream_gbps"] = g.gemm_probe_stream(dBs, scratch)
    # the same weights stored N x K (K-contiguous, a row pitch of 16 KiB): the tiles walk K in a rotated order
    dBk = dBs.t().contiguous()
    cfgk = g.gemm_select_ex(Ms, Ns, Ks, g.GEMM_BF16, g.GEMM_B_K_CONTIGUOUS)
    us = timed_us(cfgk, torch.from_numpy(As.view(np.int16)).cuda(), dBk, torch.empty((Ms, Ns), dtype=torch.int16, device="cuda"))
    also["skinny_bf16_M16_N28672_K8192_b_k_contiguous"] = {"us": us, "gbps": sk_bytes / us * 1e-3,
                                                           "frac_of_hbm_peak": sk_bytes / us * 1e-3 / PEAK_HBM_GBPS,
                                                           "picked": cfgk.describe()}
    del dBk
    # the same weight against 256 rows: still on the HBM side of the ridge (61 us of bytes, 48 us of flops at the peaks)
    Mw = 256
    dAw = torch.randn((Mw, Ks), device="cuda", generator=torch.Generator(device="cuda").manual_seed(2)).to(torch.bfloat16)
    cfgw = g.gemm_select(Mw, Ns, Ks, g.GEMM_BF16)
    us = timed_us(cfgw, dAw.view(torch.int16), dBs, torch.empty((Mw, Ns), dtype=torch.int16, device="cuda"))
    w_bytes = (Mw * Ks + Ks * Ns + Mw * Ns) * 2.0
    also["skinny_bf16_M256_N28672_K8192"] = {"us": us, "gbps": w_bytes / us * 1e-3, "frac_of_hbm_peak": w_bytes / us * 1e-3 / PEAK_HBM_GBPS,
                                             "tflops": 2.0 * Mw * Ns * Ks / us * 1e-6, "picked": cfgw.describe()}
    del dBs

    # grouped launch: 16 groups of routing-like row counts (16384 rows in all) against one 4096 x 4096
    # weight each, in one launch; beside it the same products as 16 separately selected launches
    rows = wl.routed_rows(16, 16384, seed=6)
    Ng = Kg = 4096
    shapes = [(m, Ng, Kg) for m in rows]
    Ag, Bg = wl.normal_bf16(sum(rows), Ng * 2, Kg, seed=6)          # two weights, shared alternately
    dAg = torch.from_numpy(Ag.view(np.int16)).cuda()
    dBg = [torch.from_numpy(np.ascontiguousarray(Bg[:, i * Ng:(i + 1) * Ng]).view(np.int16)).cuda() for i in range(2)]
    dCg = torch.empty((sum(rows), Ng), dtype=torch.int16, device="cuda")
    tensors, r0 = [], 0
    for i, m in enumerate(rows):
        tensors.append((dAg[r0:r0 + m], dBg[i % 2], dCg[r0:r0 + m]) if m else (None, None, None))
        r0 += m
    probs = g.make_problems(shapes, 0, tensors)
    cfg_g = g.gemm_select_grouped(probs, g.GEMM_BF16)
    table, _ = g.gemm_grouped_plan(cfg_g, probs)
    dtab = g.table_to_device(table)
    singles = [(g.gemm_select(m, Ng, Kg, g.GEMM_BF16), t) for m, t in zip(rows, tensors) if m]
    ensure_ws(max(g.gemm_workspace_bytes(c1) for c1, _ in singles))   # a single pick may split K

    def time_loop(fn):
        return settled_us(torch, fn)

    flops_g = 2.0 * sum(rows) * Ng * Kg
    us_g = time_loop(lambda: g.gemm_run_grouped(cfg_g, table, dtab))
    us_s = time_loop(lambda: [g.gemm_run(c1, *t) for c1, t in singles])
    also["grouped_bf16_16x(m,4096,4096)_16384_rows"] = {
        "tflops": flops_g / us_g * 1e-6, "us": us_g, "picked": cfg_g.describe(),
        "separate_launches_tflops": flops_g / us_s * 1e-6, "rows": rows}
    del Ag, Bg, dAg, dBg, dCg

    # the vendor library on the same box and operands (calibration of what this chip sustains on
    # N(0,1) data under its power limit; not a baseline and not part of the product path)
    try:
        a16, b16 = dev[n_big][0].view(torch.bfloat16), dev[n_big][1].view(torch.bfloat16)
        us_v = settled_us(torch, lambda: torch.matmul(a16, b16))
        also["calibration_torch_matmul_bf16_%d_tflops" % n_big] = 2.0 * n_big ** 3 / us_v * 1e-6
    except Exception as exc:   # the calibration figure is optional; the product figures above are not
        also["calibration_torch_matmul_bf16_%d_tflops" % n_big] = None
        print("bench.py: vendor calibration skipped (%s)" % exc, file=sys.stderr)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # A step takes about 1 ms.  After idling the chip first boosts, then throttles hard and needs 15-20 ms of
    # continuous work to settle at its power-limited clock (8192^3 launches: 845, 958, 1121, 1088, 1000, ...
    # back to 846 us): the warm-up has to outlast that, and the timed region is long enough to show the
    # sustained rate (it is the same over 200 and over 1000 steps).
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--brief", action="store_true", help="skip the secondary figures (for profiler runs)")
    ap.add_argument("--cpu-rows", type=int, default=8192,
                    help="rows of the 8192^3 product the CPU oracle computes for the baseline (8192: all of it, about 11 s on 16 cores)")
    ap.add_argument("--ordering", choices=("default", "no-xcd-remap", "ungrouped", "neither"), default="default",
                    help="diagnostic: run the timed steps with the XCD renumbering and / or the grouped tile order "
                         "switched off in the cfg (for counter runs that show what the rasterisation buys)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy, so that HBM byte counters "
                         "collected around this command can be scaled against a transfer of known size")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build is single-GPU by design (the paper's method excludes multi-GPU); "
                 "run with --gpus 1")

    import numpy as np
    import torch

    from paper_2512_04226_amd import binding as g
    from paper_2512_04226_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    sizes = (4096, 8192)
    host = {n: wl.config2(n) for n in sizes}
    dev = {}
    for n in sizes:
        A, B = host[n]
        dev[n] = (torch.from_numpy(A.view(np.int16)).cuda(), torch.from_numpy(B.view(np.int16)).cuda(),
                  torch.empty((n, n), dtype=torch.int16, device="cuda"))
    ws = None
    for n in sizes:
        need = g.gemm_workspace_bytes(g.gemm_select(n, n, n, g.GEMM_BF16))
        if need and (ws is None or ws.numel() * 4 < need):
            ws = torch.empty(need // 4, dtype=torch.float32, device="cuda")
            g.gemm_set_workspace(ws)

    def step(events=None):
        for n in sizes:
            cfg = g.gemm_select(n, n, n, g.GEMM_BF16)
            if args.ordering in ("no-xcd-remap", "neither"):
                cfg.xcd_remap = 0
            if args.ordering in ("ungrouped", "neither"):
                cfg.group_m = 1
            dA, dB, dC = dev[n]
            if events is not None and n == sizes[-1]:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.gemm_run(cfg, dA, dB, dC)
                e1.record()
                events.append((e0, e1))
            else:
                g.gemm_run(cfg, dA, dB, dC)

    if args.traffic_probe:
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                 # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    flops_step = sum(2.0 * n ** 3 for n in sizes)
    value = flops_step * args.steps / dt * 1e-12
    big = sizes[-1]
    kern_ms = float(np.mean([a.elapsed_time(b) for a, b in events]))
    achieved = 2.0 * big ** 3 / (kern_ms * 1e-3) * 1e-12
    cfg_big = g.gemm_select(big, big, big, g.GEMM_BF16)
    cfg_small = g.gemm_select(sizes[0], sizes[0], sizes[0], g.GEMM_BF16)

    # selector cost (host only), cf. the paper's Table II
    t1 = time.perf_counter()
    for _ in range(200):
        g.gemm_select(big, big, big, g.GEMM_BF16)
    select_us = (time.perf_counter() - t1) / 200 * 1e6

    # ---- secondary figures (outside the timed region above): per-shape rates, the fp8 and the
    # bandwidth-bound paths, and the measured ceilings both rooflines are also quoted against
    def ensure_ws(need):
        nonlocal ws
        if need and (ws is None or ws.numel() * 4 < need):
            ws = torch.empty(need // 4, dtype=torch.float32, device="cuda")
            g.gemm_set_workspace(ws)

    def timed_us(cfg, dA, dB, dC):
        ensure_ws(g.gemm_workspace_bytes(cfg))
        return settled_us(torch, lambda: g.gemm_run(cfg, dA, dB, dC))

    also = {}
    # the same step in the chip's settled state (the driver's short default run sits in the throttling transient
    # that follows an idle gap: `value` is what its flags time, this is the sustained rate)
    also["settled_value"] = flops_step / settled_us(torch, step) * 1e-6
    also["settled_8192_kernel_ms"] = settled_us(torch, lambda: g.gemm_run(cfg_big, *dev[big])) * 1e-3
    # GPU time of the warm-up steps: after an idle gap the chip needs 15-20 ms of work to settle under its power
    # limit; a timed region that starts earlier reads the transient
    warm_gpu_ms = args.warmup * ms_per_step_of(also["settled_value"], flops_step)
    also["warmup_gpu_ms"] = warm_gpu_ms
    also["value_measured_in_transient"] = bool(warm_gpu_ms < 20.0)
    if not args.brief:
        secondary(also, g, wl, np, torch, dev, sizes, timed_us, ensure_ws)

    out = {
        "metric": "GEMM TFLOP/s (bf16 in, fp32 accumulate, bf16 out; analytic kernel selection included)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "square bf16 GEMM M=N=K=4096 then 8192, row-major A and B, N(0,1) seed 1",
                   "picked_4096": cfg_small.describe(), "picked_8192": cfg_big.describe(), "ordering": args.ordering,
                   "select_us": select_us},
        "frac_of_mfma_peak": value / PEAK_TFLOPS["bf16"],
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                     "frac": achieved / PEAK_TFLOPS["bf16"], "kernel": "gemm_kernel<%s> on 8192^3" % cfg_big.describe(),
                     "avg_launch_ms": kern_ms, "traffic": read_traffic("gemm_bf16_8192_counters.txt")},
    }
    ceiling = (also.get("mfma_only_bf16_random_tflops") or {}).get("16x16x32" if cfg_big.mfma == 16 else "32x32x16")
    if ceiling:
        # against what the matrix cores alone sustain on N(0,1)-like operands under this chip's power limit
        out["roofline"]["measured_ceiling"] = ceiling
        out["roofline"]["frac_of_measured_ceiling"] = achieved / ceiling
        out["roofline"]["settled_frac"] = 2.0 * big ** 3 / (also["settled_8192_kernel_ms"] * 1e-3) * 1e-12 / PEAK_TFLOPS["bf16"]
    out["also"] = also
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host[big][0], host[big][1], args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
