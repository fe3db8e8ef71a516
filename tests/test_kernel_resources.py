"""Register budget of the compiled kernels (no GPU needed: hipcc cross-compiles and reports resource usage).
The 256x256 tiles sit at the 256-register limit of an eight-wave workgroup; a change of the K loop's source that
costs a few registers shows as scratch (spills inside the loop) long before any test of results notices."""
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_04226_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _usage(src):
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "--cuda-device-only", "-c", "-Rpass-analysis=kernel-resource-usage", "-o", os.devnull, os.path.join(CSRC, src)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    rows, cur = [], None
    for line in r.stderr.split("\n"):
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = {"name": m.group(1)}
            rows.append(cur)
        for key, pat in (("vgprs", r"VGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("waves_per_simd", r"Occupancy \[waves/SIMD\]: (\d+)")):
            m = re.search(pat, line)
            if m and cur is not None:
                cur[key] = int(m.group(1))
    return rows


def _tile(es, bm, bn, bk, wm, wn, mi, ns, bl, ft):
    """Regular expression for the whole-chunk instantiation of a tile, whatever K-loop form the table gives it."""
    return "TileI" + "".join("Li%dE" % x for x in (es, bm, bn, bk, wm, wn, mi, ns, bl, ft)) + r"Li\d+ELi0ELi0EEEEE"


@pytest.mark.skipif(shutil.which(HIPCC) is None and not os.path.exists(HIPCC), reason="needs hipcc")
def test_headline_kernels_keep_no_spills_and_no_kernel_spills_much():
    with ThreadPoolExecutor(max_workers=2) as ex:
        bf16, fp8 = ex.map(_usage, ["kernels_bf16_4.hip", "kernels_fp8_0.hip"])
    rows = bf16 + fp8
    assert len(rows) >= 40
    by_name = {r["name"]: r for r in rows}

    def find(tag):
        hit = [r for n, r in by_name.items() if re.search(tag, n)]
        assert len(hit) == 1, (tag, [n for n in by_name if "Li256ELi256" in n])
        return hit[0]

    # the picks for 8192^3: bf16 256x256x64 on a 4x2 wave grid (row-major B) and on a 2x4 grid (K-contiguous B),
    # fp8 256x256x128 on four waves
    for tag in (_tile(2, 256, 256, 64, 4, 2, 16, 2, 0, 0), _tile(2, 256, 256, 64, 2, 4, 16, 2, 1, 0),
                _tile(1, 256, 256, 128, 2, 2, 32, 2, 0, 0), _tile(1, 256, 256, 128, 2, 2, 32, 2, 1, 0)):
        r = find(tag)
        assert r["scratch"] == 0, r
    # nothing else in these files spills more than a few registers' worth
    worst = max(rows, key=lambda r: r.get("scratch", 0))
    assert worst.get("scratch", 0) <= 64, worst
