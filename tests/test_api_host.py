"""Argument checks of api.matmul that need no GPU, the sweep tool's summary of its own records, and the
calibration tool's reading of the variant table."""
import json

import pytest
import torch


def test_matmul_rejects_what_it_cannot_run_before_touching_the_gpu():
    from paper_2512_04226_amd import api, binding as g
    a = torch.zeros((8, 16), dtype=torch.bfloat16)
    b = torch.zeros((16, 8), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        api.matmul(a, b)                                   # CPU tensors
    with pytest.raises(TypeError):
        api.matmul(a.float(), b.float())                   # unsupported dtype
    with pytest.raises(TypeError):
        api.matmul(a, b.to(torch.float16))                 # mixed dtypes
    # the memoised pick is the selector's pick, for both layouts
    for layout in (g.GEMM_B_ROW_MAJOR, g.GEMM_B_K_CONTIGUOUS):
        c = api.select(300, 520, 72, g.GEMM_BF16, layout)
        ref = g.gemm_select_ex(300, 520, 72, g.GEMM_BF16, layout)
        assert bytes(c) == bytes(ref) and api.select(300, 520, 72, g.GEMM_BF16, layout) is c


def test_sweep_summary_of_records(tmp_path, capsys):
    from paper_2512_04226_amd import sweep
    rec = {"M": 64, "N": 128, "K": 256, "dtype": 0, "b_layout": 0, "n_cfgs": 3,
           "best": {"idx": 1, "cfg": "64x64x64 w2x4 mfma16 s3 split1 g8", "us": 4.0, "pred_us": 4.2},
           "pick": "64x64x64 w2x4 mfma16 s3 streamk256 g8", "pick_us": 5.0, "pick_pred_us": 4.1, "efficiency": 0.8,
           "best_tflops": 1.0, "pick_tflops": 0.8, "bottleneck": "launch", "top5": []}
    grp = {"set": "two groups", "groups": 2, "rows": [3, 4], "dtype": 0, "b_layout": 0,
           "best": {"idx": 0, "cfg": "64x64x64 w2x4 mfma16 s3 split1 g8 groups2", "us": 2.0, "pred_us": 2.0},
           "pick": "64x64x64 w2x4 mfma16 s3 split1 g8 groups2", "pick_us": 2.0, "pick_pred_us": 2.0, "efficiency": 1.0,
           "pick_tflops": 3.0, "best_tflops": 3.0, "separate_launches_us": 5.0, "top5": []}
    p1, p2 = tmp_path / "a_0.jsonl", tmp_path / "grouped.jsonl"
    p1.write_text(json.dumps(rec) + "\n")
    p2.write_text(json.dumps(grp) + "\n")
    sweep.summarize([str(p1), str(p2)])
    out = capsys.readouterr().out
    assert "a_0.jsonl" in out and "median 0.800" in out and "Stream-K picked 1, sweep-best 0" in out
    assert "grouped.jsonl (grouped)" in out and "two groups" in out and "separate launches" in out


def test_variant_table_loop_form_columns_cover_every_compiled_variant():
    """calibrate.py reprints the variant table and must carry the two K-loop-form columns over: its
    parser has to find one row per compiled variant, in table order, with a known form."""
    from paper_2512_04226_amd import binding as g, calibrate

    forms = calibrate.table_loop_forms()
    for sect, dtype in (("BF16", g.GEMM_BF16), ("FP8", g.GEMM_FP8_E4M3)):
        rows = [k for k in forms if k[0] == sect]
        assert len(rows) == g.gemm_variant_count(dtype)
        seen = set()
        for idx in range(g.gemm_cfg_count(dtype)):
            c = g.gemm_cfg_at(idx, 8192, 8192, 8192, dtype)
            if c is not None:
                seen.add((sect, c.block_m, c.block_n, c.block_k, c.waves_m, c.waves_n, c.mfma, c.stages))
        assert seen == set(rows)
    assert all(lf in range(7) and lf_kc in range(7) for lf, lf_kc in forms.values())


def test_uniform128_shapes_follow_the_papers_recipe():
    """Section V-A: dimensions are multiples of 128 up to 8192; the sample is seeded."""
    from paper_2512_04226_amd import workloads as wl

    s = wl.uniform128_shapes()
    assert len(s) == 192 and s == wl.uniform128_shapes()
    assert all(d % 128 == 0 and 128 <= d <= 8192 for shape in s for d in shape)
    assert len({d for shape in s for d in shape}) > 48          # spread over the 64 possible values
