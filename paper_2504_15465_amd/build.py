"""Build ``liblithos.so`` for gfx950 with hipcc (in-tree, no JIT cache).

    python -m paper_2504_15465_amd.build

Every translation unit under ``csrc/`` is compiled to an object file in
``csrc/_build/`` (in parallel) and linked into ``paper_2504_15465_amd/liblithos.so``.
hipcc cross-compiles, so this works on a machine without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "liblithos.so")

SOURCES = ["gemm_tile256_wide.hip", "gemm_tile256_elem.hip", "gemm_lds256_wide.hip", "gemm_lds256_elem.hip", "gemm_tile128.hip", "gemm_tile64.hip", "gemm_skinny.hip", "gemm.hip", "rowops.hip", "attention.hip", "attention_prefill.hip", "runtime.hip", "sched.hip", "sched_core.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    if src.endswith(".cpp"):
        cmd = [HIPCC, "-x", "hip"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    return obj


def _fresh(src: str) -> bool:
    """Object newer than its source and every header (only consulted by --incremental)."""
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    if not os.path.exists(obj):
        return False
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    deps.append(os.path.join(HERE, "..", "include", "lithos.h"))
    return all(os.path.getmtime(obj) > os.path.getmtime(d) for d in deps)


def build(verbose: bool = True, incremental: bool = False) -> str:
    """Compile every source (always, unless ``incremental``) and link the library."""
    os.makedirs(OBJ, exist_ok=True)
    todo = [s for s in SOURCES if not (incremental and _fresh(s))]
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as ex:
        list(ex.map(_compile, todo))
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    tmp = LIB + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs + ["-lpthread"],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    sys.exit(0)
