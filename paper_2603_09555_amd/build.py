"""Compile the HIP sources under ``csrc/`` (in-tree, gfx950 only) into two shared libraries:

* ``libssd_hip.so``      the product: every source directly under ``csrc/``;
* ``libssd_measure.so``  the same objects plus ``csrc/measure/`` (per-kernel timing of a prefill, peak
  probes): calls that create events and wait, kept out of the product library.

``hipcc`` cross-compiles without a GPU.  Every source is compiled to an object once and the objects are
linked twice.  Packed-fp32 instruction selection is disabled (``-Xclang -target-feature -Xclang
-packed-fp32-ops``) for every device translation unit.
"""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libssd_hip.so")
MEASURE_LIB = os.path.join(HERE, "libssd_measure.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def measure_sources():
    return sorted(glob.glob(os.path.join(CSRC, "measure", "*.hip")))


def needs_build() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(MEASURE_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(MEASURE_LIB))
    deps = sources() + measure_sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + \
        glob.glob(os.path.join(INCLUDE, "*.h"))
    return any(os.path.getmtime(f) > t for f in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Run hipcc.  With ``force=False`` up-to-date libraries are kept.  Returns the product library's path."""
    if not force and not needs_build():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmpdir = tempfile.mkdtemp(prefix="ssd_build_")
    try:
        def compile_one(src):
            obj = os.path.join(tmpdir, os.path.basename(src) + ".o")
            cmd = [hipcc] + HIPCC_FLAGS + ["-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), file=sys.stderr)
            subprocess.run(cmd, check=True)
            return obj

        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, sources() + measure_sources()))
        n = len(sources())
        for lib, members in ((LIB, objs[:n]), (MEASURE_LIB, objs)):
            tmp = lib + ".tmp%d" % os.getpid()
            cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + members
            if verbose:
                print(" ".join(cmd), file=sys.stderr)
            subprocess.run(cmd, check=True)
            os.replace(tmp, lib)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
