"""Offline exhaustive sweep of the compiled configuration space (evaluation tool only).

For each problem shape, times every legal (variant, split_k) configuration returned by
gemm_cfg_at plus the analytical pick of gemm_select, and records the paper's selection
efficiency (Section V-A): throughput of the pick divided by the best throughput found.
Nothing here is used by gemm_select or gemm_run.

    python -m paper_2512_04226_amd.sweep --set config5 --out sweep_config5.jsonl
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

from . import binding as g
from . import workloads as wl


def make_operands(M, N, K, dtype, seed=0, normal=False):
    """Random device operands of the right type: U[-1, 1] (config 5's values) or, with normal=True,
    N(0, 1) (config 2's).  The chip is power-limited on large compute-bound shapes, so the value
    distribution does move the timing of the big tiles by a few percent."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    if dtype in (g.GEMM_BF16, g.GEMM_FP16):
        t = torch.bfloat16 if dtype == g.GEMM_BF16 else torch.float16
        if normal:
            A = torch.randn((M, K), device="cuda", generator=gen).to(t)
            B = torch.randn((K, N), device="cuda", generator=gen).to(t)
        else:
            A = (torch.rand((M, K), device="cuda", generator=gen) * 2 - 1).to(t)
            B = (torch.rand((K, N), device="cuda", generator=gen) * 2 - 1).to(t)
    else:
        A = torch.randint(0, 0x78, (M, K), device="cuda", generator=gen, dtype=torch.uint8)
        B = torch.randint(0, 0x78, (K, N), device="cuda", generator=gen, dtype=torch.uint8)
    C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
    return A, B, C


class Workspace:
    def __init__(self):
        self.t = None

    def ensure(self, cfg):
        need = g.gemm_workspace_bytes(cfg)
        if need and (self.t is None or self.t.numel() * 4 < need):
            self.t = torch.empty((need + 3) // 4, dtype=torch.float32, device="cuda")
            g.gemm_set_workspace(self.t)


def time_cfg(cfg, A, B, C, ws, min_ms=1.0, max_iters=200, repeats=3):
    """Microseconds per launch: `iters` back-to-back launches captured in a HIP graph (so
    that host launch overhead does not mask short kernels), replayed `repeats` times between
    events on torch's current stream; the median replay is reported."""
    ws.ensure(cfg)
    return time_launch(lambda: g.gemm_run(cfg, A, B, C), min_ms, max_iters, repeats)


def time_launch(launch, min_ms=1.0, max_iters=200, repeats=3):
    """The timing protocol of time_cfg for any enqueueing callable."""
    launch()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    launch()
    e1.record()
    e1.synchronize()
    one = max(e0.elapsed_time(e1), 1e-3)
    iters = int(min(max_iters, max(3, min_ms / one)))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(iters):
            launch()
    graph.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(repeats):
        e0.record()
        graph.replay()
        e1.record()
        e1.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / iters)
    del graph
    return float(np.median(times))


def sweep_shape(M, N, K, dtype, ws, quick=False, b_layout=0):
    A, B, C = make_operands(M, N, K, dtype)
    flops = 2.0 * M * N * K
    rows = []
    for idx in range(g.gemm_cfg_count(dtype)):
        cfg = g.gemm_cfg_at_ex(idx, M, N, K, dtype, b_layout)
        if cfg is None:
            continue
        us = time_cfg(cfg, A, B, C, ws, min_ms=0.5 if quick else 1.0)
        rows.append({"idx": idx, "cfg": cfg.describe(), "us": us, "pred_us": cfg.predicted_us})
    # Finalists: the five fastest of the first pass and the analytic pick.  All of them are timed again,
    # the same number of times, round-robin (so that drift of the chip's state hits all alike), and each
    # keeps the median of its timings: the pick gets no second chance that the others do not get.
    pick = g.gemm_select_ex(M, N, K, dtype, b_layout)
    by_cfg = {r["cfg"]: r for r in rows}
    finalists = sorted(rows, key=lambda r: r["us"])[:5]
    if pick.describe() not in [r["cfg"] for r in finalists]:
        finalists.append(by_cfg[pick.describe()])
    cfgs = {r["cfg"]: g.gemm_cfg_at_ex(r["idx"], M, N, K, dtype, b_layout) for r in finalists}
    again = {r["cfg"]: [r["us"]] for r in finalists}
    for _ in range(2):
        for r in finalists:
            again[r["cfg"]].append(time_cfg(cfgs[r["cfg"]], A, B, C, ws))
    final = [dict(r, us=float(np.median(again[r["cfg"]]))) for r in finalists]
    best = min(final, key=lambda r: r["us"])
    pick_us = [r["us"] for r in final if r["cfg"] == pick.describe()][0]
    rec = {"M": M, "N": N, "K": K, "dtype": dtype, "b_layout": b_layout, "n_cfgs": len(rows), "best": best, "pick": pick.describe(),
           "pick_us": pick_us, "pick_pred_us": pick.predicted_us, "efficiency": min(1.0, best["us"] / pick_us),
           "best_tflops": flops / best["us"] * 1e-6, "pick_tflops": flops / pick_us * 1e-6,
           "bottleneck": g.BOTTLENECKS[pick.bottleneck],
           "top5": sorted(final, key=lambda r: r["us"])[:5]}
    return rec, rows


def rerank(paths):
    """Offline: what the selector as it stands now would have scored on recorded sweeps (files written with
    --all-rows).  For every recorded shape the present gemm_select pick is looked up among the recorded
    timings of all configurations; efficiency = fastest recorded time / the pick's recorded time, one timing
    each, capped at 1.  No GPU is used."""
    for path in paths:
        recs = [json.loads(line) for line in open(path) if line.strip()]
        effs, missing = [], 0
        for r in recs:
            if "rows" not in r:
                missing += 1
                continue
            pick = g.gemm_select_ex(r["M"], r["N"], r["K"], r["dtype"], r.get("b_layout", 0)).describe()
            us = {x["cfg"]: x["us"] for x in r["rows"]}
            if pick not in us:
                missing += 1
                continue
            effs.append(min(1.0, min(us.values()) / us[pick]))
        if effs:
            print("%-40s n=%3d  median %.3f  mean %.3f  min %.3f  >=0.95: %d%s" % (
                os.path.basename(path), len(effs), np.median(effs), np.mean(effs), np.min(effs), sum(e >= 0.95 for e in effs),
                "  (%d shapes without a recorded timing of the pick)" % missing if missing else ""))
        else:
            print("%-40s no record with all rows" % os.path.basename(path))


def grouped_sets():
    """Grouped workloads: routing-like row counts against per-group weights, and one mixed list."""
    return [
        ("16 routed x 4096x4096", [(m, 4096, 4096) for m in wl.routed_rows(16, 16384, seed=6)]),
        ("8 routed x 4096x2048", [(m, 4096, 2048) for m in wl.routed_rows(8, 4096, seed=11)]),
        ("64 routed x 2048x1024", [(m, 2048, 1024) for m in wl.routed_rows(64, 8192, seed=5, skew=0.5)]),
        ("32 routed x 1024x7168", [(m, 1024, 7168) for m in wl.routed_rows(32, 2048, seed=12, skew=0.3)]),
        ("128 routed x 7168x2048", [(m, 7168, 2048) for m in wl.routed_rows(128, 1024, seed=13)]),
        ("8 routed x 2048x7168 (65536 rows)", [(m, 2048, 7168) for m in wl.routed_rows(8, 65536, seed=14)]),
        ("16 equal x 256x4096x4096", [(256, 4096, 4096)] * 16),
        ("mixed", [(4096, 4096, 4096), (512, 8192, 1024), (2048, 1024, 8192), (64, 14336, 4096)]),
    ]


def sweep_grouped(name, shapes, dtype, b_layout=0):
    """Every variant's grouped launch and the analytic pick on one group list; the same groups as
    separately selected launches for reference."""
    ws = Workspace()
    tensors = []
    for i, (M, N, K) in enumerate(shapes):
        if M == 0:
            tensors.append((None, None, None))
            continue
        A, B, C = make_operands(M, N, K, dtype, seed=i)
        tensors.append((A, B.t().contiguous() if b_layout else B, C))
    probs = g.make_problems(shapes, b_layout, tensors)
    flops = sum(2.0 * M * N * K for (M, N, K) in shapes)

    def timed(cfg):
        table, _ = g.gemm_grouped_plan(cfg, probs)
        dtab = g.table_to_device(table)
        return time_launch(lambda: g.gemm_run_grouped(cfg, table, dtab))

    rows = []
    for vid in range(g.gemm_variant_count(dtype)):
        cfg = g.gemm_cfg_at_grouped(vid, probs, dtype, b_layout)
        if cfg is None:
            continue
        rows.append({"idx": vid, "cfg": cfg.describe(), "us": timed(cfg), "pred_us": cfg.predicted_us})
    pick = g.gemm_select_grouped(probs, dtype, b_layout)
    # one timing each: the pick is one of the rows
    pick_us = [r for r in rows if r["idx"] == pick.kernel_id][0]["us"]
    best = min(rows, key=lambda r: r["us"])
    singles = [(g.gemm_select_ex(M, N, K, dtype, b_layout), t) for (M, N, K), t in zip(shapes, tensors) if M]
    for c1, _ in singles:
        ws.ensure(c1)
    sep_us = time_launch(lambda: [g.gemm_run(c1, *t) for c1, t in singles])
    return {"set": name, "groups": len(shapes), "rows": [s[0] for s in shapes], "dtype": dtype, "b_layout": b_layout,
            "best": best, "pick": pick.describe(), "pick_us": pick_us, "pick_pred_us": pick.predicted_us,
            "efficiency": min(1.0, best["us"] / pick_us), "pick_tflops": flops / pick_us * 1e-6,
            "best_tflops": flops / best["us"] * 1e-6, "separate_launches_us": sep_us,
            "top5": sorted(rows, key=lambda r: r["us"])[:5]}


def summarize(paths):
    """Text summary of sweep records (the JSONL files this tool wrote): one line per file with the
    selection efficiency, then one line per shape."""
    dt_name = {g.GEMM_BF16: "bf16", g.GEMM_FP8_E4M3: "fp8", g.GEMM_FP16: "fp16"}
    heads, body = [], []
    for path in paths:
        recs = [json.loads(line) for line in open(path) if line.strip()]
        if not recs:
            continue
        if "set" in recs[0]:      # grouped records
            e = [r["efficiency"] for r in recs]
            heads.append("%-52s n=%2d  median %.3f  mean %.3f  min %.3f  >=0.95: %d" % (
                os.path.basename(path) + " (grouped)", len(e), np.median(e), np.mean(e), np.min(e), sum(x >= 0.95 for x in e)))
            for r in recs:
                tag = " groups%d" % r["groups"]
                body.append("%-36s | %-44s %8.1f | %-44s %8.1f | %5.3f | %7.1f | separate launches %8.1f us" % (
                    r["set"], r["pick"].replace(tag, ""), r["pick_us"], r["best"]["cfg"].replace(tag, ""), r["best"]["us"],
                    r["efficiency"], r["pick_tflops"], r["separate_launches_us"]))
            continue
        e = [r["efficiency"] for r in recs]
        n_cfg = [r["n_cfgs"] for r in recs]
        heads.append("%-52s n=%2d  median %.3f  mean %.3f  min %.3f  >=0.95: %d  configs/shape %d..%d  Stream-K picked %d, sweep-best %d" % (
            os.path.basename(path), len(e), np.median(e), np.mean(e), np.min(e), sum(x >= 0.95 for x in e), min(n_cfg),
            max(n_cfg), sum("streamk" in r["pick"] for r in recs), sum("streamk" in r["best"]["cfg"] for r in recs)))
        for r in recs:
            body.append("%6d %6d %6d %-4s L%d | %-44s %8.1f | %-44s %8.1f | %5.3f | %7.1f" % (
                r["M"], r["N"], r["K"], dt_name[r["dtype"]], r.get("b_layout", 0), r["pick"], r["pick_us"], r["best"]["cfg"],
                r["best"]["us"], r["efficiency"], r["pick_tflops"]))
    print("\n".join(heads))
    print("\nPer shape (M N K dtype layout | pick | pick us | sweep best | best us | efficiency | pick TFLOP/s):")
    print("\n".join(body))


def shape_set(name):
    if name == "config5":
        return [(m, n, k, g.GEMM_BF16) for (m, n, k) in wl.config5_shapes()]
    if name == "square":
        return [(n, n, n, g.GEMM_BF16) for n in (512, 1024, 2048, 4096, 8192)]
    if name == "skinny":
        return [(m, n, k, g.GEMM_BF16) for (n, k) in wl.SKINNY_NK for m in wl.SKINNY_M]
    if name == "fp8":
        return [(n, n, n, g.GEMM_FP8_E4M3) for n in (1024, 4096, 8192)]
    if name == "fp16":      # the paper's precision; run with --b-layout 1 for its operand layout too
        return [(n, n, n, g.GEMM_FP16) for n in (1024, 2048, 4096, 8192)] + [(4864, 4096, 4096, g.GEMM_FP16)]
    if name == "uniform128":    # the shape distribution and precision of the paper's Section V-A; --b-layout 1 for its layout
        return [(m, n, k, g.GEMM_FP16) for (m, n, k) in wl.uniform128_shapes()]
    if name == "uniform128fp8":  # the same distribution (first 96 shapes) in fp8 e4m3
        return [(m, n, k, g.GEMM_FP8_E4M3) for (m, n, k) in wl.uniform128_shapes()[:96]]
    raise SystemExit("unknown shape set " + name)


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--set", default="config5")
    ap.add_argument("--out", default="sweep.jsonl")
    ap.add_argument("--limit", type=int, default=0)
    ap.add_argument("--quick", action="store_true")
    ap.add_argument("--b-layout", type=int, default=0, help="0: B row-major K x N, 1: B stored K-contiguous (N x K)")
    ap.add_argument("--all-rows", action="store_true", help="also write every config's timing")
    ap.add_argument("--summarize", nargs="+", metavar="JSONL", help="print a text summary of sweep records and exit")
    ap.add_argument("--rerank", nargs="+", metavar="JSONL",
                    help="score the present selector on recorded sweeps (written with --all-rows); needs no GPU")
    args = ap.parse_args(argv)
    if args.summarize:
        summarize(args.summarize)
        return
    if args.rerank:
        rerank(args.rerank)
        return
    if args.set == "grouped":
        os.makedirs(os.path.dirname(args.out) or ".", exist_ok=True)
        effs = []
        with open(args.out, "a") as f:
            for name, shapes in grouped_sets():
                rec = sweep_grouped(name, shapes, g.GEMM_BF16, args.b_layout)
                f.write(json.dumps(rec) + "\n")
                f.flush()
                effs.append(rec["efficiency"])
                print("%s: best %s %.1f us, pick %s %.1f us (pred %.1f) eff %.3f, %.0f TF; separate launches %.1f us" % (
                    name, rec["best"]["cfg"], rec["best"]["us"], rec["pick"], rec["pick_us"], rec["pick_pred_us"],
                    rec["efficiency"], rec["pick_tflops"], rec["separate_launches_us"]), flush=True)
        print("grouped selection efficiency: median %.3f mean %.3f min %.3f over %d group lists" % (
            float(np.median(effs)), float(np.mean(effs)), float(np.min(effs)), len(effs)), flush=True)
        return
    shapes = shape_set(args.set)
    if args.limit:
        shapes = shapes[:args.limit]
    done = set()
    if os.path.exists(args.out):       # resume: skip shapes already recorded
        for line in open(args.out):
            try:
                r = json.loads(line)
                if r.get("b_layout", 0) == args.b_layout:
                    done.add((r["M"], r["N"], r["K"], r["dtype"]))
            except ValueError:
                pass
    os.makedirs(os.path.dirname(args.out) or ".", exist_ok=True)
    ws = Workspace()
    effs = []
    with open(args.out, "a") as f:
        for i, (M, N, K, dt) in enumerate(shapes):
            if (M, N, K, dt) in done:
                continue
            t0 = time.time()
            rec, rows = sweep_shape(M, N, K, dt, ws, quick=args.quick, b_layout=args.b_layout)
            if args.all_rows:
                rec["rows"] = rows
            f.write(json.dumps(rec) + "\n")
            f.flush()
            effs.append(rec["efficiency"])
            print("[%d/%d] %dx%dx%d best %s %.1f us (%.0f TF) pick %s %.1f us eff %.3f  (%.1fs)" % (
                i + 1, len(shapes), M, N, K, rec["best"]["cfg"], rec["best"]["us"], rec["best_tflops"], rec["pick"],
                rec["pick_us"], rec["efficiency"], time.time() - t0), flush=True)
    if effs:
        print("selection efficiency: median %.3f mean %.3f min %.3f over %d shapes" % (
            float(np.median(effs)), float(np.mean(effs)), float(np.min(effs)), len(effs)), flush=True)


if __name__ == "__main__":
    main()
