"""Device calibration of the model's constants (a one-off, offline step; never run by
gemm_select or gemm_run):

  * L_MI of every matrix instruction, the MFMA ceiling on workload-like operands, the L2, MALL and HBM
    read rates, the LDS fragment-read rates and the load latency, from the library's probes;
  * the measured cost of a K slab of every kernel variant (steady-state clocks per slab of one tile on a
    full CU, from one large compute-bound problem per datatype, 8192^3) beside the compute latency the
    model assigns it from the descriptor alone (Algorithm 3's L_MT plus the slab's fill and synchronisation
    cost): the data the two fitted constants fill_issue_bytes_per_clk and slab_sync_clk come from.  No
    per-variant timing enters the selector.

Prints the descriptor fields the probes give and one line per variant (B row-major and K-contiguous).

    python -m paper_2512_04226_amd.calibrate [--n 8192]

The K-loop form of each variant (LOOP / LOOP_KC columns) is chosen from a comparison of
builds of the library, one per form (0 .. 6), each with that form forced on every variant (a tile that
does not fit form 6 runs form 0 in that build):

    for k in 0 1 2 3 4 5 6: python -m paper_2512_04226_amd.build --out /tmp/lf$k.so -DG355_FORCE_LOOP_FORM=$k
    python -m paper_2512_04226_amd.calibrate --loop-forms /tmp/lf0.so /tmp/lf1.so /tmp/lf2.so /tmp/lf3.so /tmp/lf4.so /tmp/lf5.so /tmp/lf6.so

which ends with the table rows carrying the chosen forms.
"""
import argparse
import ctypes
import os
import re

import numpy as np
import torch

from . import binding as g
from .sweep import Workspace, make_operands


def _table(first, last):
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "variants.hpp")
    out, sect = {}, "BF16"
    for line in open(path):
        m = re.match(r"#define G355_VARIANTS_(BF16|FP8)_\d", line)
        if m:
            sect = m.group(1)
        m = re.match(r"\s*X\(" + ", ".join([r"(\d+)"] * 9) + r"\)", line)
        if m:
            v = [int(x) for x in m.groups()]
            out[(sect,) + tuple(v[:7])] = tuple(v[first:last])
    return out


def table_loop_forms():
    """(section, block_m, block_n, block_k, waves_m, waves_n, mfma, stages) -> (LOOP, LOOP_KC) as
    written in csrc/variants.hpp, in table order."""
    return _table(7, 9)


def measure_rates():
    """Every entry of the hardware descriptor that the device itself can report, from the library's probes:
    L_MI per matrix instruction, the MFMA ceiling on constant and on workload-like operands, the L2, MALL
    and HBM read rates, the LDS fragment-read rates and the load latency at each level."""
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
            out[(name, mi, "settled")] = (g.gemm_probe_mfma_ex(dt, mi, 0, scratch), g.gemm_probe_mfma_ex(dt, mi, 1, scratch))
    per_clk = 1.0 / hw.clk_ghz                                                # GB/s -> bytes per clock
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)     # 1 GiB > MALL
    out["hbm_gbps"] = g.gemm_probe_stream(buf, scratch)
    # repeated reads: 16 MiB stays in the eight L2s (2 MiB each), 128 MiB in the MALL, 1 GiB in neither
    out["l2_gbps"] = g.gemm_probe_read(buf[:16 << 20], 64, scratch)
    out["mall_gbps"] = g.gemm_probe_read(buf[:128 << 20], 8, scratch)
    out["hbm_repeat_gbps"] = g.gemm_probe_read(buf, 2, scratch)
    for kind, name in enumerate(("lds_b128", "lds_b64", "lds_tr_b16", "lds_tr_b8")):
        by_waves = {w: g.gemm_probe_lds(kind, w, scratch) for w in (4, 8, 16)}
        for w, x in by_waves.items():
            out["%s_%dwaves_gbps" % (name, w)] = x
        out[name + "_gbps"] = max(by_waves.values())
    # the refill path by itself: 64 KiB slabs towards LDS from data that the L2s, the MALL or HBM hold
    for kind, kname in ((0, "direct"), (2, "registers"), (3, "registers_ds_write")):
        out["fill_%s_l2_gbps" % kname] = g.gemm_probe_fill(kind, 1, buf, 2048, scratch, sync=1)
        out["fill_%s_mall_gbps" % kname] = g.gemm_probe_fill(kind, 2, buf, 128 << 20, scratch, sync=1)
        out["fill_%s_hbm_gbps" % kname] = g.gemm_probe_fill(kind, 2, buf, 1 << 30, scratch, sync=1)
    out["lat_l2_ns"] = g.gemm_probe_latency(buf[:2 << 20], scratch)
    out["lat_mall_ns"] = g.gemm_probe_latency(buf[:128 << 20], scratch)
    out["lat_hbm_ns"] = g.gemm_probe_latency(buf, scratch)
    out["gemm_hw"] = {
        "hbm_bytes_per_clk": out["hbm_gbps"] * per_clk,
        "mall_bytes_per_clk": out["mall_gbps"] * per_clk,
        "l2_bytes_per_clk": out["l2_gbps"] * per_clk / hw.n_xcd,
        "lds_bytes_per_clk": out["lds_b128_gbps"] * per_clk / hw.n_cu,
        "lds_tr_bytes_per_clk": out["lds_tr_b16_gbps"] * per_clk / hw.n_cu,
        "mem_latency_clk": out["lat_hbm_ns"] * hw.clk_ghz,
        "l_mi_clk": [[out[("bf16", 32)][1], out[("bf16", 16)][1]], [out[("fp8", 32)][1], out[("fp8", 16)][1]]],
    }
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


def compare_loop_forms(lib_paths, n=8192, passes=7):
    """Times every variant of every datatype and B layout in each of the given builds of the
    library (the same cfg, plain launches, the builds and variants interleaved in shuffled
    passes, median) and prints one line per variant: microseconds per build and the ratios to
    the first.  The outputs of the builds are compared bit for bit first."""
    libs = [ctypes.CDLL(p) for p in lib_paths]
    for lib in libs:
        lib.gemm_run.restype = ctypes.c_int

    def run(lib, cfg, A, B, C):
        rc = lib.gemm_run(ctypes.byref(cfg), g._ptr(A), g._ptr(B), g._ptr(C), ctypes.c_void_p(g._stream_handle(None)))
        if rc != 0:
            raise RuntimeError("gemm_run returned %d" % rc)

    def time_one(lib, cfg, A, B, C, launches=6):
        for _ in range(2):
            run(lib, cfg, A, B, C)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(launches):
            run(lib, cfg, A, B, C)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / launches

    rng = np.random.default_rng(1)
    ratios = {}
    for dtype, name in ((g.GEMM_BF16, "bf16"), (g.GEMM_FP16, "fp16"), (g.GEMM_FP8_E4M3, "fp8")):
        for bl in (0, 1):
            A, B, C = make_operands(n, n, n, dtype, normal=True)
            if bl:
                B = B.t().contiguous()
            cfgs, seen = [], set()
            for idx in range(g.gemm_cfg_count(dtype)):
                c = g.gemm_cfg_at_ex(idx, n, n, n, dtype, bl)
                if c is None or c.split_k != 1 or c.stream_k or c.kernel_id in seen:
                    continue
                seen.add(c.kernel_id)
                cfgs.append(c)
            for c in cfgs:
                outs = []
                for lib in libs:
                    C.zero_()
                    run(lib, c, A, B, C)
                    torch.cuda.synchronize()
                    outs.append(C.clone())
                if any(not torch.equal(outs[0], o) for o in outs[1:]):
                    raise RuntimeError("builds disagree on " + c.describe())
            times = {(c.kernel_id, i): [] for c in cfgs for i in range(len(libs))}
            for _ in range(passes):
                order = [(c, i) for c in cfgs for i in range(len(libs))]
                rng.shuffle(order)
                for c, i in order:
                    times[(c.kernel_id, i)].append(time_one(libs[i], c, A, B, C))
            for c in cfgs:
                med = [float(np.median(times[(c.kernel_id, i)])) for i in range(len(libs))]
                print("%s b_layout %d variant %-3d %-44s us %s  vs first %s" % (
                    name, bl, c.kernel_id, c.describe(), " ".join("%8.1f" % x for x in med),
                    " ".join("%.3f" % (x / med[0]) for x in med)), flush=True)
                key = (c.block_m, c.block_n, c.block_k, c.waves_m, c.waves_n, c.mfma, c.stages)
                ratios.setdefault(("FP8" if dtype == g.GEMM_FP8_E4M3 else "BF16", bl) + key, []).append(
                    [x / med[0] for x in med])
    # the table's choice: build i is form i; bf16 and fp16 share the 16-bit list, so their ratios are
    # averaged; a form other than 0 must be at least 1.5 % faster than form 0 to be taken
    def choice(sect, bl, key):
        mean = np.mean(np.array(ratios[(sect, bl) + key]), axis=0)
        best = int(np.argmin(mean))
        return best if mean[best] < 0.985 else 0

    print("// LOOP / LOOP_KC columns chosen from the timings above (other columns as in the table)")
    for full in table_loop_forms():
        sect, key = full[0], full[1:]
        print("%s    X(%s, %d, %d)" % (sect, ", ".join(str(x) for x in key), choice(sect, 0, key), choice(sect, 1, key)),
              flush=True)


def decompose(lib_paths, n=8192):
    """Where a K slab's time goes: the large tiles of each datatype on n^3, timed in a normal build and in the
    timing-only diagnostic builds without the refills, without the fragment reads, and without both
    (LIB_FULL LIB_SKIP_FILL LIB_SKIP_FRAG LIB_SKIP_BOTH, all built with the same forced K-loop form), on
    N(0,1)-like and on all-zero operands (the latter take the power limit out of the picture)."""
    names = ("full", "no fill", "no fragment reads", "neither")
    libs = [ctypes.CDLL(p) for p in lib_paths]
    for lib in libs:
        lib.gemm_run.restype = ctypes.c_int

    def settled(lib, cfg, A, B, C):
        def run():
            if lib.gemm_run(ctypes.byref(cfg), g._ptr(A), g._ptr(B), g._ptr(C), ctypes.c_void_p(g._stream_handle(None))) != 0:
                raise RuntimeError("gemm_run failed")
        for _ in range(40):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(30):
            run()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / 30

    picks = {g.GEMM_BF16: ("256x256x64 w2x4 mfma16 s2 split1 ", "256x256x64 w2x4 mfma32 s2 split1 ", "256x256x32 w2x4 mfma32 s4 split1 ",
                           "256x256x32 w2x4 mfma32 s5 split1 ", "256x128x64 w2x4 mfma16 s3 split1 ", "128x128x64 w2x4 mfma16 s2 split1 ",
                           "128x128x64 w2x4 mfma16 s4 split1 "),
             g.GEMM_FP8_E4M3: ("256x256x128 w2x4 mfma32 s2 split1 ", "128x128x128 w2x2 mfma32 s2 split1 ")}
    for dtype, label in ((g.GEMM_BF16, "bf16"), (g.GEMM_FP8_E4M3, "fp8")):
        for zeros in (False, True):
            A, B, C = make_operands(n, n, n, dtype, normal=True)
            if zeros:
                A.zero_()
                B.zero_()
            for idx in range(g.gemm_cfg_count(dtype)):
                c = g.gemm_cfg_at(idx, n, n, n, dtype)
                if c is None or not c.describe().startswith(picks[dtype]):
                    continue
                us = [settled(lib, c, A, B, C) for lib in libs]
                print("%-4s %-8s %-38s %s" % (label, "zeros" if zeros else "random", c.describe(), "   ".join(
                    "%s %.0f us (%.0f TFLOP/s)" % (nm, t, 2.0 * n ** 3 / t * 1e-6) for nm, t in zip(names, us))), flush=True)


def compare_builds(named_libs, n=8192):
    """The large tiles of each datatype on n^3 in several builds of the library (NAME=PATH each; the
    timing-only diagnostic builds of gemm_kernel.hpp among them), settled, N(0,1)-like operands."""
    libs = []
    for a in named_libs:
        name, path = a.split("=", 1)
        lib = ctypes.CDLL(path)
        lib.gemm_run.restype = ctypes.c_int
        libs.append((name, lib))

    def settled(lib, cfg, A, B, C):
        def run():
            if lib.gemm_run(ctypes.byref(cfg), g._ptr(A), g._ptr(B), g._ptr(C), ctypes.c_void_p(g._stream_handle(None))) != 0:
                raise RuntimeError("gemm_run failed")
        for _ in range(30):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            run()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / 20

    picks = {g.GEMM_BF16: ("256x256x64 w4x2 mfma16 s2 split1 ", "256x256x64 w2x4 mfma16 s2 split1 ", "256x256x32 w2x4 mfma32 s4 split1 ",
                           "128x128x64 w2x4 mfma16 s2 split1 ", "128x128x64 w2x4 mfma16 s4 split1 ", "256x128x64 w2x4 mfma16 s3 split1 "),
             g.GEMM_FP8_E4M3: ("256x256x128 w2x4 mfma32 s2 split1 ",)}
    for dtype, label in ((g.GEMM_BF16, "bf16"), (g.GEMM_FP8_E4M3, "fp8")):
        A, B, C = make_operands(n, n, n, dtype, normal=True)
        for idx in range(g.gemm_cfg_count(dtype)):
            c = g.gemm_cfg_at(idx, n, n, n, dtype)
            if c is None or not c.describe().startswith(picks[dtype]):
                continue
            print("%-4s %-40s %s" % (label, c.describe(), "  ".join("%s %.0f us" % (nm, settled(l, c, A, B, C)) for nm, l in libs)),
                  flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=8192)
    ap.add_argument("--skip-rates", action="store_true")
    ap.add_argument("--rates-only", action="store_true", help="run the probes, print the descriptor fields, stop")
    ap.add_argument("--loop-forms", nargs="+", metavar="LIB",
                    help="compare builds of the library (one per forced K-loop form) instead of calibrating")
    ap.add_argument("--decompose", nargs=4, metavar="LIB",
                    help="time the large tiles in four builds: normal, -DG355_DIAG_SKIP_FILL, -DG355_DIAG_SKIP_FRAG, both")
    ap.add_argument("--compare-builds", nargs="+", metavar="NAME=LIB",
                    help="time the large tiles in each of several builds of the library (diagnostic builds among them)")
    args = ap.parse_args()
    if args.compare_builds:
        compare_builds(args.compare_builds, args.n)
        return
    if args.decompose:
        decompose(args.decompose, args.n)
        return
    if args.loop_forms:
        compare_loop_forms(args.loop_forms, args.n)
        return
    if not args.skip_rates:
        r = measure_rates()
        for key, val in r.items():
            if key == "gemm_hw":
                print("gemm_hw fields from the probes (bytes per %.1f GHz clock):" % g.gemm_hw_get().clk_ghz)
                for f, x in val.items():
                    print("    %-22s %s" % (f, ("%.1f" % x) if not isinstance(x, list) else
                                            "[[%.1f, %.1f], [%.1f, %.1f]]" % (x[0][0], x[0][1], x[1][0], x[1][1])))
            elif isinstance(key, str):
                print("%-18s %.1f" % (key, val))
            elif len(key) == 3:
                print("MFMA %s %dx%d settled: %.0f TFLOP/s on constant operands, %.0f on workload-like operands" % (
                    key[0], key[1], key[1], val[0], val[1]))
            else:
                print("MFMA %s %dx%d: %.0f TFLOP/s device-wide -> L_MI = %.1f clk" % (key[0], key[1], key[1], val[0], val[1]))
        if args.rates_only:
            return
    for dtype, name in ((g.GEMM_BF16, "BF16"), (g.GEMM_FP8_E4M3, "FP8")):
        print("// %s variants on %d^3: measured clocks per slab | the model's compute latency per slab (L_MT + fill + sync)" % (name, args.n))
        rows = measure_slab_clk(dtype, args.n, 0)
        rows_kc = measure_slab_clk(dtype, args.n, 1)
        for (cfg, us, tau), (_, us_kc, tau_kc) in zip(rows, rows_kc):
            p = g.gemm_predict(cfg)
            model = p.l_compute / max(1, p.occupancy)
            print("    %-36s measured %5.0f (K-contiguous B %5.0f)  model %5.0f  ratio %.2f   // %.1f us %.0f TFLOP/s | %.1f us %.0f TFLOP/s" % (
                cfg.describe(), tau, tau_kc, model, tau / model, us, 2.0 * args.n ** 3 / us * 1e-6, us_kc,
                2.0 * args.n ** 3 / us_kc * 1e-6), flush=True)


if __name__ == "__main__":
    main()
