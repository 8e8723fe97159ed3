"""Builds librlstm.so (HIP, gfx950 only) in-tree with hipcc.

Every source is compiled to an object file under _build/ (several at a time), then linked.
`python paper_1608_00895_amd/build.py --incremental` recompiles only sources that are newer than
their object file (or older than a header); build() without it compiles everything.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librlstm.so")
SOURCES = ["gemm.hip", "recurrent.hip", "recurrent_persistent.hip", "recurrent_stepwise.hip", "exchange_probe.hip",
           "mdlstm.hip", "mdlstm_stepwise.hip", "chunking.hip", "output_layer.hip", "stream.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fvisibility=hidden",
    # packed fp32 VALU forms are not used on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def _headers_mtime() -> float:
    hs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    return max(os.path.getmtime(h) for h in hs)


def build(verbose: bool = True, incremental: bool = False, jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hm = _headers_mtime()
    todo = []
    objs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s + ".o")
        objs.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hm)
        if not (incremental and fresh):
            todo.append([HIPCC] + FLAGS + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(run, todo))
    run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden"] + objs + ["-o", LIB])
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv)
    print("built", LIB)
