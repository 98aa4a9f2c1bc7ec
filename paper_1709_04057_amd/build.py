"""Builds liblinrec.so (HIP, gfx950 only) next to this file.

One hipcc invocation per translation unit, run in parallel: the tile kernels are compiled once per
tile shape (-DLINREC_TILE_ID=n), then everything is linked into one shared library.  Each HIP unit
is compiled in a directory of its own with the intermediate files kept, so that the device assembly
of exactly the code that is linked can be checked (see isa_check.py) before the rest is deleted.
"""
from __future__ import annotations

import glob
import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

try:
    from . import isa_check
except ImportError:  # run as a script
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import isa_check

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.environ.get("LINREC_BUILD_OUT", os.path.join(HERE, "liblinrec.so"))
OBJ_DIR = os.environ.get("LINREC_BUILD_DIR", os.path.join(HERE, "_build"))

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC] + os.environ.get("LINREC_EXTRA_FLAGS", "").split()


def tile_ids():
    with open(os.path.join(CSRC, "linrec_launch.h")) as f:
        return [int(m) for m in re.findall(r"^\s*X\((\d+),", f.read(), flags=re.M)]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def _compile_hip(job):
    """Compiles one HIP unit, checks its device assembly, keeps the object file only."""
    src, extra, obj = job
    work = os.path.join(OBJ_DIR, obj[:-2] + ".tmp")
    shutil.rmtree(work, ignore_errors=True)
    os.makedirs(work)
    tmp_obj = os.path.join(work, obj)
    out = _run([HIPCC] + FLAGS + extra + ["-save-temps=obj", "-c", os.path.join(CSRC, src), "-o", tmp_obj])
    asm = glob.glob(os.path.join(work, "*-hip-amdgcn-amd-amdhsa-gfx950.s"))
    if len(asm) != 1:
        raise RuntimeError("%s: expected one device assembly file, found %r" % (obj, asm))
    with open(asm[0]) as f:
        problems = isa_check.check_text(f.read(), obj[:-2] + ".s")
    if problems:
        raise RuntimeError("device assembly check failed for %s (%s):\n%s" % (obj, " ".join(extra), "\n".join(problems[:20])))
    os.replace(tmp_obj, os.path.join(OBJ_DIR, obj))
    shutil.rmtree(work, ignore_errors=True)
    return out


def _compile_host(job):
    src, _, obj = job
    return _run(["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", "-I" + os.path.join(ROOT, "include"),
                 "-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ_DIR, obj)])


def build(verbose: bool = False, jobs: int | None = None) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    units = [("linrec_api.hip", [], "api.o"), ("linrec_scan.hip", [], "scan.o"),
             ("linrec_validate.cpp", ["-x", "c++"], "validate.o")]
    for i in tile_ids():
        units.append(("linrec_tiles.hip", ["-DLINREC_TILE_ID=%d" % i], "tile_%d.o" % i))
    jobs = jobs or min(8, os.cpu_count() or 4)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for out in ex.map(lambda u: (_compile_host if u[0].endswith(".cpp") else _compile_hip)(u), units):
            if verbose and out.strip():
                print(out)
    objs = [os.path.join(OBJ_DIR, o) for _, _, o in units]
    tmp = LIB + ".tmp.%d" % os.getpid()
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
