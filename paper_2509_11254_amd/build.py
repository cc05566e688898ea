"""Build libpsgd.so (gfx950) from csrc/ with hipcc, in-tree.  `python -m paper_2509_11254_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpsgd.so")
CEIL_LIB = os.path.join(HERE, "libpsgd_ceilings.so")      # plain streaming kernels for `bench.py --ceilings`
SOURCES = ["api.hip", "prod.hip", "form.hip", "residual.hip", "thin.hip"]
CEIL_SOURCE = "ceilings.hip"
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-sanitize",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr[-4000:]))
    return obj


def build(verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES + [CEIL_SOURCE]))
    for lib, parts in ((LIB, objs[:-1]), (CEIL_LIB, objs[-1:])):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *parts]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n%s" % res.stderr[-4000:])
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
