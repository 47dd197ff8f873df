"""Builds libpre3.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpre3.so")
SOURCES = ["grammar.cpp", "lr1.cpp", "tables.cpp", "token_edges.cpp", "symbol_edges.cpp", "api.cpp",
           "mask_kernels.hip", "apply_kernels.hip", "sampler_kernels.hip", "advance_kernels.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the host pass does not know the packed-fp32 target feature and says so: harmless
_NOISE = "is not a recognized feature for this target"


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in proc.stderr.splitlines() if _NOISE not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]) + "\n" + err)
    return err


def _newest_header() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    paths.append(os.path.join(HERE, "..", "include", "pre3.h"))
    return max(os.path.getmtime(p) for p in paths)


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compiles every source to an object (in parallel) and links the shared library.  With
    `incremental` an object newer than its source and every header is kept."""
    os.makedirs(OBJ, exist_ok=True)
    newest_h = _newest_header()
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_h)
        if not (incremental and fresh):
            jobs.append(["hipcc", *FLAGS, "-c", "-o", obj, src])
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        notes = list(pool.map(_run, jobs))
    notes.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", LIB,
                       *[os.path.join(OBJ, s + ".o") for s in SOURCES]]))
    if verbose:
        print("\n".join(n for n in notes if n.strip()))
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
