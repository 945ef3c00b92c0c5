"""Builds (hipcc, gfx950) and runs the microbenchmarks on the current GPU:

    python -m paper_2206_01288_amd.microbench            # issue rates
    python -m paper_2206_01288_amd.microbench gather     # gather rate

Issue rates: per instruction kind, number of independent chains and wavefronts per SIMD, the time per launch, the
time per instruction per wavefront and the shader-clock ticks per instruction of one wavefront. Gather rate: the
cycles a CU spends per 64-lane gather from a table row, by entry size and order of the columns.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
BUILD = os.path.join(os.path.dirname(HERE), "_build")


def build():
    """Compiles the microbenchmarks for gfx950 and returns the paths of the executables by name."""
    os.makedirs(BUILD, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    exes = {}
    for name in ("issue_rates", "gather_rate"):
        exes[name] = os.path.join(BUILD, name)
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                               "-packed-fp32-ops", "-Wno-unused-value", os.path.join(HERE, name + ".hip"), "-o", exes[name]])
    return exes


def main():
    exes = build()
    if "--build-only" in sys.argv:
        return
    sys.exit(subprocess.call([exes["gather_rate" if "gather" in sys.argv else "issue_rates"]]))


if __name__ == "__main__":
    main()
