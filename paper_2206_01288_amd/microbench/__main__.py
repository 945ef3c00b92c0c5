"""Builds (hipcc, gfx950) and runs the issue-rate microbenchmark on the current GPU:

    python -m paper_2206_01288_amd.microbench

Prints, per instruction kind, number of independent chains and wavefronts per SIMD, the time per launch, the
time per instruction per wavefront and the shader-clock ticks per instruction of one wavefront.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
BUILD = os.path.join(os.path.dirname(HERE), "_build")


def build():
    """Compiles issue_rates.hip for gfx950 and returns the path of the executable."""
    os.makedirs(BUILD, exist_ok=True)
    exe = os.path.join(BUILD, "issue_rates")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-Wno-unused-value", os.path.join(HERE, "issue_rates.hip"), "-o", exe])
    return exe


def main():
    exe = build()
    if "--build-only" in sys.argv:
        return
    sys.exit(subprocess.call([exe]))


if __name__ == "__main__":
    main()
