"""Build libemc2.so (HIP, gfx950 only) in-tree with hipcc: one object per source, compiled in parallel, then linked."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libemc2.so")
PROBE_LIB = os.path.join(HERE, "libemc2probe.so")     # measurement probes of the bench (include/emc2_probe.h)
SOURCES = ["context.hip", "cellindex.hip", "voxelize.hip", "kmap.hip", "spconv.hip", "spconv_mfma.hip", "spconv_span.hip",
           "spconv_direct.hip", "project.hip", "decoder.hip", "pool.hip", "dispatch.hip", "spconv_i8.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


def _headers_mtime() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + [os.path.join(ROOT, "include", "emc2.h")]
    return max(os.path.getmtime(h) for h in hs)


def build(verbose: bool = False, force: bool = True, jobs: int = 8) -> str:
    """force=True recompiles every source; force=False only those newer than their object (or older than a header)."""
    os.makedirs(OBJ, exist_ok=True)
    hm = _headers_mtime()

    def compile_one(src: str) -> str:
        s, o = os.path.join(CSRC, src), os.path.join(OBJ, src + ".o")
        if not force and os.path.exists(o) and os.path.getmtime(o) > max(os.path.getmtime(s), hm):
            return o
        cmd = ["hipcc"] + FLAGS + ["-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return o

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, SOURCES + ["probes.hip"]))
    for lib, members in ((LIB, objs[:-1]), (PROBE_LIB, objs[-1:])):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + members
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, force="--incremental" not in sys.argv))
