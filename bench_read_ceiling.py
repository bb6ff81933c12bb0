#!/usr/bin/env python3
"""Read ceiling of the decode kernel's work decomposition: builds and runs the stand-alone microbenchmark
paper_2509_06261_amd/csrc/read_ceiling.hip (kernels that only load: the decode kernel's persistent waves and tiles,
and a plain sequential read by short-lived workgroups) and prints its table.  A measurement aid beside bench.py; the
library does not depend on it.

  python bench_read_ceiling.py [pool GiB = 128] [32 KiB chunks per wave = 192] [workgroups = 512] [group = 8]
  python bench_read_ceiling.py --build-only        (compile here, run later on the GPU machine)
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(ROOT, "paper_2509_06261_amd", "csrc", "read_ceiling.hip")
EXE = os.path.join(ROOT, "paper_2509_06261_amd", "read_ceiling")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build():
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wall", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", SRC, "-o", EXE], check=True, stderr=subprocess.DEVNULL)


def main():
    args = [a for a in sys.argv[1:] if a != "--build-only"]
    if "--build-only" in sys.argv or not os.path.exists(EXE) or os.path.getmtime(EXE) < os.path.getmtime(SRC):
        build()
    if "--build-only" in sys.argv:
        return 0
    return subprocess.run([EXE, *(args or ["128", "192", "512", "8"])]).returncode


if __name__ == "__main__":
    sys.exit(main())
