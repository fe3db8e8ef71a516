"""Build the gfx950 shared library in-tree (hipcc for the kernels, g++ for the host-only
selector).  Usage: python -m paper_2512_04226_amd.build [-f]
With --out LIB [-DNAME=VALUE ...] it builds a second library with extra kernel defines
somewhere else, e.g. the builds `calibrate.py --loop-forms` compares:
  python -m paper_2512_04226_amd.build --out /tmp/lf0.so -DG355_FORCE_LOOP_FORM=0"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libgemm355.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra"]


def _sources():
    hip = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    host = sorted(f for f in os.listdir(CSRC) if f.endswith(".cpp"))
    return hip, host


def _deps_mtime():
    return max(os.path.getmtime(os.path.join(CSRC, f)) for f in os.listdir(CSRC)
               if f.endswith((".hpp", ".inc", ".h"))) if os.path.isdir(CSRC) else 0


def _compile(src, force, obj_dir=None, defines=()):
    obj = os.path.join(obj_dir or OBJ, src + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(path), _deps_mtime(),
                 os.path.getmtime(os.path.join(PKG, "..", "include", "gemm.h")))
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj, False
    if src.endswith(".hip"):
        cmd = [HIPCC] + HIP_FLAGS + list(defines) + ["-c", path, "-o", obj]
    else:
        cmd = ["g++"] + HOST_FLAGS + ["-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), r.stderr))
    return obj, True


def build(force=False, jobs=8, out=None, defines=()):
    """out / defines: build another library (always from scratch, objects beside it) with extra
    -D options for the kernels; the in-tree library is the default."""
    lib = os.path.abspath(out) if out else LIB
    obj_dir = lib + ".obj" if out else OBJ
    force = force or bool(out)
    os.makedirs(obj_dir, exist_ok=True)
    hip, host = _sources()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        res = list(ex.map(lambda s: _compile(s, force, obj_dir, defines), hip + host))
    objs = [o for o, _ in res]
    if force or any(changed for _, changed in res) or not os.path.exists(lib):
        tmp = lib + ".%d.tmp" % os.getpid()
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed: %s\n%s" % (" ".join(cmd), r.stderr))
        os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    argv = sys.argv[1:]
    print(build(force="-f" in argv, out=argv[argv.index("--out") + 1] if "--out" in argv else None,
                defines=[a for a in argv if a.startswith("-D")]))
