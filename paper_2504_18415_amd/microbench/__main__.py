"""Builds and runs the chip-ceiling micro-benchmarks (needs a GPU): python -m paper_2504_18415_amd.microbench"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def build() -> str:
    exe = os.path.join(HERE, "chip_ceilings")
    src = os.path.join(HERE, "chip_ceilings.hip")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-Wno-unused-command-line-argument", src, "-o", exe], check=True,
                   stderr=subprocess.DEVNULL)
    return exe


if __name__ == "__main__":
    exe = build()
    if "--build-only" not in sys.argv:
        sys.exit(subprocess.run([exe]).returncode)
