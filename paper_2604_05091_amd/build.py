"""Build libmegatrain_mi355.so (gfx950) in-tree with hipcc.

    python -m paper_2604_05091_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmegatrain_mi355.so")
SOURCES = ["gemm.hip", "elementwise.hip", "attention.hip", "engine.cpp", "kernels_api.cpp", "host_ops.cpp"]
HOST_ONLY = {"host_ops.cpp"}  # no device code: plain g++ (function multi-versioning for the Adam loop)
HEADERS = ["common.h", "host_ops.h", "../../include/megatrain.h", "../../include/megatrain_kernels.h"]
# -packed-fp32-ops off: the compiler must not form packed fp32 instructions on this target
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-result", "-x", "hip"]


def _newest(paths):
    return max(os.path.getmtime(p) for p in paths)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hdr_time = _newest([os.path.join(CSRC, h) for h in HEADERS])
    jobs = []
    objs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src + ".o")
        objs.append(o)
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), hdr_time):
            if src in HOST_ONLY:
                jobs.append(["g++", "-O3", "-std=c++17", "-fPIC", "-pthread", "-c", s, "-o", o])
            else:
                jobs.append(["hipcc", *FLAGS, "-c", s, "-o", o])

    def run(cmd):
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(run, jobs))
    if jobs or force or not os.path.exists(LIB):
        run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-lpthread"])
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
