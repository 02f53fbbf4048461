"""Build the HIP libraries of this package for gfx950, in-tree.

`python -m paper_2003_00822_amd.build` compiles `csrc/*.hip` into
`paper_2003_00822_amd/libpbatch.so` with hipcc (cross-compiles without a GPU):
one object per source, compiled in parallel, then one link; and the calibration
loop of the benchmark (`csrc/calib/`, not part of the product) into
`paper_2003_00822_amd/libpbatch_calib.so`.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpbatch.so")
CALIB_LIB = os.path.join(HERE, "libpbatch_calib.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 VALU forms are not to be generated on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]
# Per-source flags.  The product kernel's leading scalar arguments (the ones its first memory requests need) are
# preloaded into registers by the hardware when a wave starts; the compiler keeps a fallback entry that loads them
# for firmware without the feature.
FILE_FLAGS = {
    "pb_mfma.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=12"],
}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def calib_sources():
    return sorted(glob.glob(os.path.join(CSRC, "calib", "*.hip")))


def _compile(src: str, extra, verbose: bool) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".%d.o" % os.getpid())
    cmd = [HIPCC] + FLAGS + FILE_FLAGS.get(os.path.basename(src), []) + list(extra) + ["-c", "-o", obj, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return obj


def build(verbose: bool = True, extra_flags=(), out: str = LIB, srcs=None) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources() if srcs is None else srcs
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        objs = list(pool.map(lambda s: _compile(s, extra_flags, verbose), srcs))
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    try:
        subprocess.check_call(cmd)
        os.replace(tmp, out)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    return out


def build_all(verbose: bool = True):
    return [build(verbose), build(verbose, out=CALIB_LIB, srcs=calib_sources())]


if __name__ == "__main__":
    for lib in build_all():
        print("built", lib)
    sys.exit(0)
