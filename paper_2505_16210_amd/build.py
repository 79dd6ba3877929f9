"""Builds libnqkv.so (the C-ABI library with the gfx950 kernels) and libnqkv_benchaux.so (the
benchmark's measurement helpers) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnqkv.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
          # keep the compiler from forming packed-fp32 instructions
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-function"]
# (source, extra flags).  The quantizer and dequantizer define stored bits: no contraction.
SOURCES = [
    ("nqkv_host.cpp", ["-x", "hip", "-ffp-contract=off"]),
    ("quantize.hip", ["-ffp-contract=off"]),
    ("dequantize.hip", ["-ffp-contract=off"]),
    ("decode_attention.hip", []),
    ("decode_multi.hip", []),
    ("static_scratch.hip", []),
]
TIMELINE_LIB = os.path.join(HERE, "libnqkv_timeline.so")      # measurement build, see build_timeline_library
AUX_LIB = os.path.join(HERE, "libnqkv_benchaux.so")
AUX_SOURCES = [("bench_aux.hip", [])]


def _compile(src: str, extra: list, verbose: bool, save_temps: bool, tag: str = "") -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + tag + ".o")
    cmd = [HIPCC, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    if save_temps:
        cmd.append("--save-temps=obj")
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=OBJ)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops" not in l)      # the host pass does not know the feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return obj


def build_library(verbose: bool = False, save_temps: bool = False, jobs: int = 4) -> str:
    os.makedirs(OBJ, exist_ok=True)
    # the translation units are independent: compile them side by side (a few hipcc processes,
    # each a few hundred MB)
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(lambda se: _compile(se[0], se[1], verbose, save_temps), SOURCES + AUX_SOURCES))
    for lib, lib_objs in ((LIB, objs[:len(SOURCES)]), (AUX_LIB, objs[len(SOURCES):])):
        tmp = lib + ".tmp.%d" % os.getpid()
        cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *lib_objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        os.replace(tmp, lib)
    return LIB


def build_timeline_library(verbose: bool = False) -> str:
    """libnqkv_timeline.so: the library with the decode kernel compiled -DNQKV_TIMELINE (every wave
    leaves eight timestamps of its item in the workspace).  For `bench.py --timeline` only; needs
    the objects of build_library()."""
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s, _ in SOURCES if s != "decode_attention.hip"]
    if not all(os.path.exists(o) for o in objs):
        build_library(verbose=verbose)
    objs.append(_compile("decode_attention.hip", ["-DNQKV_TIMELINE"], verbose, False, tag="_timeline"))
    tmp = TIMELINE_LIB + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, TIMELINE_LIB)
    return TIMELINE_LIB


if __name__ == "__main__":
    print(build_library(verbose=True, save_temps="--save-temps" in sys.argv))
    if "--timeline" in sys.argv:
        print(build_timeline_library(verbose=True))
