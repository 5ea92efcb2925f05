"""Builds libcorr_mi355x.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libcorr_mi355x.so")
OBJ_DIR = os.path.join(PKG, "_build")
# (source, object name, extra flags); block.hip is built once per lookup radius
SOURCES = [("corr_api.hip", "corr_api.o", []), ("features.hip", "features.o", []), ("binning.hip", "binning.o", []),
           ("ondemand.hip", "ondemand.o", []), ("fullvol.hip", "fullvol.o", []), ("backward.hip", "backward.o", [])]
SOURCES += [("block.hip", "block_r%d.o" % r, ["-DCORR_BLOCK_R=%d" % r]) for r in (4, 3, 2, 1)]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-I" + INCLUDE, "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]
FLAGS += os.environ.get("CORR_EXTRA_HIPCC_FLAGS", "").split()   # for experiments only


def _compile(job) -> str:
    src, objname, extra = job
    obj = os.path.join(OBJ_DIR, objname)
    cmd = [HIPCC] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        print(err)
    return obj


def build_library(verbose: bool = True) -> str:
    """Compile every HIP source and link the shared library (always rebuilds)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
