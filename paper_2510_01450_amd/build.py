"""Builds the C-ABI library from csrc/*.hip with hipcc for gfx950, in-tree.

Two artefacts from the same sources:
  libllla.so          the production library (include/llla.h);
  libllla_measure.so  the same sources compiled with -DLLLA_MEASURE (kernel launchers record HIP events) plus
                      csrc/measure/*.hip (include/llla_measure.h) -- loaded by the benchmark only.
Each gets a stamp file holding a hash of the sources it was built from; the binding compares it before loading.
"""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllla.so")
LIB_MEASURE = os.path.join(HERE, "libllla_measure.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Wall", "-Wno-unused-function",
    # packed fp32 ALU forms are switched off for all device code of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def sources(measure: bool = False):
    src = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    if measure:
        src += sorted(glob.glob(os.path.join(CSRC, "measure", "*.hip")))
    return src


def source_hash(measure: bool = False) -> str:
    """Hash of everything a library is compiled from (sources, headers, flags)."""
    h = hashlib.sha256()
    files = sources(measure) + sorted(glob.glob(os.path.join(CSRC, "*.hpp"))) + sorted(
        glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.relpath(f, ROOT).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(FLAGS[:-2]).encode())
    return h.hexdigest()


def stamp_path(lib: str) -> str:
    return lib + ".stamp"


def is_current(lib: str, measure: bool = False) -> bool:
    """True when `lib` exists and was built from the sources as they are now."""
    try:
        with open(stamp_path(lib)) as fh:
            return os.path.exists(lib) and fh.read().strip() == source_hash(measure)
    except OSError:
        return False


def _build_one(lib: str, measure: bool, verbose: bool, extra) -> str:
    bdir = os.path.join(HERE, "_build", "measure" if measure else "product")
    os.makedirs(bdir, exist_ok=True)
    procs, objs = [], []
    for src in sources(measure):
        obj = os.path.join(bdir, os.path.basename(src) + ".o")
        cmd = [HIPCC] + FLAGS + (["-DLLLA_MEASURE"] if measure else []) + list(extra) + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd)))
        objs.append(obj)
    failed = [src for src, pr in procs if pr.wait() != 0]
    if failed:
        raise RuntimeError("hipcc failed for: " + ", ".join(failed))
    tmp = lib + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    with open(stamp_path(lib), "w") as fh:
        fh.write(source_hash(measure) + "\n")
    return lib


def build(verbose: bool = False, extra=(), measure: bool = True) -> str:
    """Compile every HIP source into libllla.so (and libllla_measure.so).  Always recompiles."""
    _build_one(LIB, False, verbose, extra)
    if measure:
        _build_one(LIB_MEASURE, True, verbose, extra)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
