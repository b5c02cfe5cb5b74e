"""Build libhbp.so (C-ABI library: HIP kernels for gfx950 + host planner) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libhbp.so")
LIB_RACE_HUNT = os.path.join(PKG, "libhbp_racehunt.so")   # the same library with a full fence after every phase
OBJ_DIR = os.path.join(PKG, "_build")
SOURCES = ["api.hip", "fwd.hip", "bwd.hip", "loss.hip", "plan.cpp", "balance.cpp", "auto_select.cpp"]

HIP_FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-munsafe-fp-atomics", "-Wno-inline-asm",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", INCLUDE, "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str, race_hunt: bool = False) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + (".racehunt.o" if race_hunt else ".o"))
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        cmd = [_hipcc()] + HIP_FLAGS + (["-DHBP_RACE_HUNT"] if race_hunt else []) + ["-c", path, "-o", obj]
    else:
        cmd = ["g++", "-O2", "-fPIC", "-std=c++17", "-I", INCLUDE, "-c", path, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), out))
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def _link(objs, lib: str) -> None:
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    os.replace(tmp, lib)


def build_library(verbose: bool = True, race_hunt: bool = True) -> str:
    """Compile every source and link libhbp.so; always rebuilds.  race_hunt: also libhbp_racehunt.so, the
    attention kernels with a workgroup fence after every phase (a test compares the two bit for bit)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    fenced = [s for s in ("fwd.hip", "bwd.hip") if race_hunt]
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
        objs_rh = list(ex.map(lambda s: _compile(s, True), fenced))
    _link(objs, LIB)
    if race_hunt:
        by_src = dict(zip(fenced, objs_rh))
        _link([by_src.get(s, o) for s, o in zip(SOURCES, objs)], LIB_RACE_HUNT)
    if verbose:
        print("built", LIB + (" and " + LIB_RACE_HUNT if race_hunt else ""))
    return LIB


if __name__ == "__main__":
    build_library()
