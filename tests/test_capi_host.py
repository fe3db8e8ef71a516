"""Host-side checks of the C ABI: every declared symbol is exported, argument validation
returns the documented codes, the selector is deterministic and needs no GPU."""
import ctypes
import os
import re
import threading

import pytest

from paper_2512_04226_amd import binding as g

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "gemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gemm_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"gemm_select", "gemm_run", "gemm_workspace_bytes", "gemm_set_workspace", "gemm_cfg_count",
            "gemm_cfg_at", "gemm_predict", "gemm_hw_get", "gemm_hw_set", "gemm_hw_reset", "gemm_hw_preset", "gemm_strerror",
            "gemm_abi_version"} <= set(names)
    lib = ctypes.CDLL(g.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
        assert callable(getattr(g, n, None)), "the binding has no function named %s" % n
    assert g.gemm_abi_version() == g.GEMM_ABI_VERSION


def test_struct_layouts_match_the_header(tmp_path):
    """Compile the public header with gcc and compare sizeof / offsetof of every field with the
    binding's ctypes structures."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lines = ["#include <stdio.h>", "#include <stddef.h>", '#include "gemm.h"', "int main(void){"]
    structs = {"gemm_cfg": g.gemm_cfg, "gemm_prediction": g.gemm_prediction, "gemm_hw": g.gemm_hw,
               "gemm_sk_segment": g.gemm_sk_segment, "gemm_problem": g.gemm_problem,
               "gemm_group_rec": g.gemm_group_rec}
    for name, cls in structs.items():
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (name, name))
        for field, _ in cls._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (name, field, name, field))
    lines.append("return 0;}")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(root, "include"), "-o", str(exe), str(src)])
    got = dict(line.split() for line in subprocess.check_output([str(exe)], text=True).splitlines())
    for name, cls in structs.items():
        assert int(got[name]) == ctypes.sizeof(cls), name
        for field, _ in cls._fields_:
            assert int(got["%s.%s" % (name, field)]) == getattr(cls, field).offset, (name, field)
    assert ctypes.sizeof(g.gemm_cfg) == 136 and ctypes.sizeof(g.gemm_group_rec) == 64


def test_select_argument_errors():
    cfg = g.gemm_cfg()
    f = g._lib.gemm_select
    assert f(512, 512, 512, 0, None) == -1                     # NULL out
    assert f(0, 512, 512, 0, ctypes.byref(cfg)) == -2          # shape
    assert f(512, -1, 512, 0, ctypes.byref(cfg)) == -2
    assert f(512, 512, 512, 7, ctypes.byref(cfg)) == -3        # dtype
    # selection is total on M, N, K >= 1; the default leading dimensions are rounded up to 16 bytes
    assert f(512, 516, 512, 0, ctypes.byref(cfg)) == 0 and (cfg.lda, cfg.ldb, cfg.ldc) == (512, 520, 520)
    assert f(512, 512, 520, 1, ctypes.byref(cfg)) == 0 and (cfg.lda, cfg.ldb, cfg.ldc) == (528, 512, 512)
    assert f(1, 8, 8, 0, ctypes.byref(cfg)) == 0
    assert f(1, 1, 1, 0, ctypes.byref(cfg)) == 0 and (cfg.lda, cfg.ldb, cfg.ldc) == (8, 8, 8)   # smallest problem
    assert f(5, 1, 7, 1, ctypes.byref(cfg)) == 0 and (cfg.lda, cfg.ldb, cfg.ldc) == (16, 16, 8)
    assert g._lib.gemm_select_ex(33, 1001, 72, 0, 1, ctypes.byref(cfg)) == 0 and (cfg.lda, cfg.ldb, cfg.ldc) == (72, 72, 1008)
    assert f(1 << 31, 512, 512, 0, ctypes.byref(cfg)) == -2
    for code in range(0, -10, -1):
        assert g.gemm_strerror(code) != "unknown status"
    assert g.gemm_strerror(-99) == "unknown status"


def test_cfg_at_enumeration_and_legality():
    n = g.gemm_cfg_count(g.GEMM_BF16)
    assert 75 <= n <= 400 and g.gemm_cfg_count(g.GEMM_FP8_E4M3) >= 50
    assert g._lib.gemm_cfg_count(5) == -3
    cfg = g.gemm_cfg()
    assert g._lib.gemm_cfg_at(-1, 512, 512, 512, 0, ctypes.byref(cfg)) == -9
    assert g._lib.gemm_cfg_at(n, 512, 512, 512, 0, ctypes.byref(cfg)) == -9
    legal = [g.gemm_cfg_at(i, 512, 512, 64, 0) for i in range(n)]
    # K = 64 has one or two slabs: no variant may split it 32 ways
    assert all(c is None or c.split_k <= 2 for c in legal) and any(c is not None for c in legal)
    seen = set()
    for i in range(n):
        c = g.gemm_cfg_at(i, 4096, 4096, 8192, 0)
        if c is None:
            # only a stream-K entry may be illegal here: the tile count has no partial wave to split
            assert i % 7 == 6
            continue
        assert c.abi_version == g.GEMM_ABI_VERSION and c.M == 4096 and c.lda == 8192 and c.ldb == 4096
        assert (c.stream_k == 1) == (i % 7 == 6) and (c.sk_workers > 0) == (c.stream_k == 1)
        assert c.block_k % (16 if c.mfma == 32 else 32) == 0 and c.k_unroll == c.block_k // (16 if c.mfma == 32 else 32)
        assert c.stages * (c.block_m + c.block_n) * c.block_k * 2 <= 160 * 1024
        seen.add((c.kernel_id, c.split_k, c.stream_k))
    assert n - n // 7 <= len(seen) <= n and any(k[2] for k in seen)


def test_run_rejects_bad_arguments_without_launching():
    cfg = g.gemm_select(512, 512, 512, g.GEMM_BF16)
    run = g._lib.gemm_run
    p = ctypes.c_void_p(0x1000)     # never dereferenced: every case fails validation first
    assert run(None, p, p, p, None) == -1
    assert run(ctypes.byref(cfg), None, p, p, None) == -1
    bad = cfg.copy(); bad.abi_version = 99
    assert run(ctypes.byref(bad), p, p, p, None) == -7
    bad = cfg.copy(); bad.kernel_id = 10_000
    assert run(ctypes.byref(bad), p, p, p, None) == -4
    bad = cfg.copy(); bad.block_m = bad.block_m + 16
    assert run(ctypes.byref(bad), p, p, p, None) == -4
    bad = cfg.copy(); bad.split_k = 4096
    assert run(ctypes.byref(bad), p, p, p, None) == -4
    bad = cfg.copy(); bad.group_m = 0
    assert run(ctypes.byref(bad), p, p, p, None) == -4
    bad = cfg.copy(); bad.lda = 256
    assert run(ctypes.byref(bad), p, p, p, None) == -2
    bad = cfg.copy(); bad.ldb = 516
    assert run(ctypes.byref(bad), p, p, p, None) == -5
    assert run(ctypes.byref(cfg), ctypes.c_void_p(0x1008), p, p, None) == -5
    bad = cfg.copy(); bad.dtype = 9
    assert run(ctypes.byref(bad), p, p, p, None) == -3
    assert g.gemm_workspace_bytes(cfg) == (0 if cfg.split_k == 1 else cfg.split_k * 512 * 512 * 4)


def test_select_is_deterministic_and_thread_safe():
    shapes = [(512, 512, 512), (4096, 4096, 4096), (16, 28672, 8192), (1, 8192, 28672), (1808, 7344, 272)]
    ref = {s: bytes(g.gemm_select(*s, g.GEMM_BF16)) for s in shapes}
    out = []

    def worker():
        for _ in range(20):
            for s in shapes:
                out.append(bytes(g.gemm_select(*s, g.GEMM_BF16)) == ref[s])

    ts = [threading.Thread(target=worker) for _ in range(4)]
    [t.start() for t in ts]
    [t.join() for t in ts]
    assert all(out) and len(out) == 4 * 20 * len(shapes)


def test_hw_descriptor_roundtrip_and_retarget():
    hw = g.gemm_hw_get()
    assert hw.n_cu == 256 and hw.n_xcd == 8 and hw.lds_bytes == 160 * 1024 and hw.l2_bytes == 4 << 20
    try:
        small = g.gemm_hw_get()
        small.n_cu, small.n_xcd = 64, 2          # a quarter of the chip: fewer CUs -> more waves for the same tiles
        g.gemm_hw_set(small)
        p_small = g.gemm_predict(g.gemm_cfg_at(0, 8192, 8192, 8192, 0))
        g.gemm_hw_reset()
        p_full = g.gemm_predict(g.gemm_cfg_at(0, 8192, 8192, 8192, 0))
        assert p_small.waves == 4 * p_full.waves and p_small.total_us > 3 * p_full.total_us
        bad = g.gemm_hw_get(); bad.n_cu = 0
        with pytest.raises(g.GemmError):
            g.gemm_hw_set(bad)
    finally:
        g.gemm_hw_reset()
    assert bytes(g.gemm_hw_get()) == bytes(hw)


def test_small_and_skinny_problems_do_not_get_one_giant_tile():
    # Section II-A: a 256x256 output with one 256x256 tile would use a single CU
    c = g.gemm_select(256, 256, 8192, g.GEMM_BF16)
    tiles = -(-256 // c.block_m) * -(-256 // c.block_n) * c.split_k
    assert tiles >= 32, c.describe()
    for M in (1, 16, 64):
        c = g.gemm_select(M, 28672, 8192, g.GEMM_BF16)
        # bandwidth-bound: rows of a tile beyond M cost matrix-core time that is hidden under the
        # stream of B, but never a 256-row tile, and enough workgroups to keep every CU loading
        assert c.block_m <= (64 if M <= 16 else 128), c.describe()
        assert -(-28672 // c.block_n) * c.split_k >= 112, c.describe()
    c = g.gemm_select(512, 512, 512, g.GEMM_BF16)
    assert not (c.block_m == 256 and c.block_n == 256 and c.split_k == 1)


def test_run_rejects_operand_windows_of_2_gib_and_more():
    """The kernel addresses a tile's operands with 32-bit byte offsets: leading dimensions that put a
    tile's A rows, or B's K extent, 2 GiB apart must be refused before any launch."""
    run = g._lib.gemm_run
    p = ctypes.c_void_p(0x1000)
    cfg = g.gemm_select(256, 8192, 8192, g.GEMM_BF16)
    # only rejected configurations are passed to gemm_run here: nothing may reach a launch with these pointers
    bad = cfg.copy(); bad.lda = (1 << 31) // (2 * bad.block_m)       # block_m rows * lda * 2 bytes = 2 GiB
    assert run(ctypes.byref(bad), p, p, p, None) == -2
    k_slice = -(-8192 // cfg.split_k)                                 # B's window spans one K slice
    bad = cfg.copy(); bad.ldb = ((1 << 31) // (2 * k_slice) + 7) // 8 * 8  # K-slice rows * ldb * 2 bytes >= 2 GiB
    assert run(ctypes.byref(bad), p, p, p, None) == -2
    kc = g.gemm_select_ex(256, 8192, 8192, g.GEMM_BF16, g.GEMM_B_K_CONTIGUOUS)
    bad = kc.copy(); bad.ldb = (1 << 31) // (2 * bad.block_n)
    assert run(ctypes.byref(bad), p, p, p, None) == -2
    assert g._lib.gemm_select((1 << 30) + 8, 8, 8, 0, ctypes.byref(cfg)) == -2
