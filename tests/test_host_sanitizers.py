"""The selector's host code (capi.cpp + model.cpp) under ASan and UBSan on random shapes."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_selector_host_code_is_clean_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    csrc = os.path.join(ROOT, "paper_2512_04226_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(ROOT, "tests", "host_fuzz.cpp"),
           os.path.join(csrc, "capi.cpp"), os.path.join(csrc, "model.cpp")]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitize" in build.stderr:
        pytest.skip("sanitizer runtime not available: " + build.stderr[-200:])
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and run.stdout.startswith("ok"), (run.stdout[-500:], run.stderr[-2000:])
