"""Builds libdtfm.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2206_01288_amd.build [--force]

Objects go to paper_2206_01288_amd/_build/, the library to paper_2206_01288_amd/libdtfm.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libdtfm.so")

# -ffp-contract=off: every written fp64 operation rounds once (no FMA fusion), which the bit-exact
# comparison with the CPU oracle relies on. The -target-feature flag keeps the compiler from
# forming packed-fp32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Per-file additions. The fused 64-device kernels are long straight-line register programmes; the
# default scheduler orders them for low register pressure, which leaves every packed 16-bit result
# one wait state away from its consumer. The ILP-first strategy interleaves the independent chains.
_ILP = ["-mllvm", "-amdgpu-sched-strategy=iterative-ilp"]
FILE_FLAGS = {"dtfm_fast64.hip": _ILP, "dtfm_fast64_allpairs.hip": _ILP}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _newest_dep():
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "dtfm.h")]
    return max(os.path.getmtime(d) for d in deps)


def build(force: bool = False, verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("DTFM_EXTRA_HIPCC_FLAGS", "").split()
    dep_time = _newest_dep()
    jobs = []
    objs = []
    for src in sources():
        obj = os.path.join(OBJ, src[:-4] + ".o")
        objs.append(obj)
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < dep_time:
            jobs.append([hipcc] + FLAGS + FILE_FLAGS.get(src, []) + extra + ["-c", os.path.join(CSRC, src), "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(run, jobs))
    if jobs or force or not os.path.exists(LIB):
        tmp = LIB + ".tmp%d" % os.getpid()
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv)
