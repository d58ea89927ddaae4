"""Compile libmlip.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmlip.so")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# graph.hip holds the fp64 edge predicate and slab rule, whose operation order is fixed: no FMA contraction
SOURCES = {"api.hip": [], "graph.hip": ["-ffp-contract=off"], "model.hip": []}


def build(verbose=False, defines=(), lib=LIB, build_dir=BUILD):
    """defines: extra -D macros (timing experiments, e.g. MLIP_TIMING_SKIP_PAIR_PHASE); such a build goes to another
    `lib` path, never to the library the binding loads."""
    os.makedirs(build_dir, exist_ok=True)

    def compile_one(item):
        src, extra = item
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        cmd = ["hipcc", *COMMON, *extra, *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 or verbose:
            sys.stderr.write(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}")
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES.items()))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    return lib


if __name__ == "__main__":
    # python -m paper_2506_02023_amd.build [-v] [-DNAME ... --out PATH]
    defs = [a[2:] for a in sys.argv[1:] if a.startswith("-D")]
    out = sys.argv[sys.argv.index("--out") + 1] if "--out" in sys.argv else LIB
    if defs and out == LIB:
        sys.exit("a build with extra defines needs --out PATH (it must not replace the product library)")
    print(build(verbose="-v" in sys.argv, defines=defs, lib=out, build_dir=BUILD if out == LIB else BUILD + "_exp"))
