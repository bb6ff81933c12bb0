"""Builds libfineserve.so (hipcc, gfx950) next to this file."""
from __future__ import annotations

import os
import subprocess

_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_DIR)
LIB = os.path.join(_DIR, "libfineserve.so")
SOURCES = ["fs_pool.hip", "fs_append.hip", "fs_attention.hip", "fs_attention_generic.hip", "fs_attention_mfma.hip",
           "fs_prefill.hip", "fs_sched.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -packed-fp32-ops off: the compiler must not form packed fp32 instructions.
# -ffp-contract=off: quantizer arithmetic must not be fused (bytes are compared bit for bit).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
FLAGS += os.environ.get("FS_EXTRA_HIPCC_FLAGS", "").split()  # experiments only
# The prefill kernels keep MFMA accumulators and results in vector registers (no AccVGPR operands): their softmax
# reads every S^T tile with the vector ALU, which cannot address AccVGPRs.
FILE_FLAGS = {"fs_prefill.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


TIMELINE_LIB = os.path.join(_DIR, "libfineserve_timeline.so")


def build(verbose: bool = False, timeline: bool = False) -> str:
    """The library; timeline=True: its profiling twin libfineserve_timeline.so (-DFS_TIMELINE: the decode kernel
    leaves clock readings at the end of the workspace; what bench_timeline.py loads, never the product path)."""
    csrc = os.path.join(_DIR, "csrc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(csrc, src.replace(".hip", ".timeline.o" if timeline else ".o"))
        cmd = [HIPCC, *FLAGS, *(["-DFS_TIMELINE"] if timeline else []), *FILE_FLAGS.get(src, []), "-I",
               os.path.join(ROOT, "include"), "-I", csrc, "-c", os.path.join(csrc, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(ln for ln in out.splitlines() if "packed-fp32-ops" not in ln)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    lib = TIMELINE_LIB if timeline else LIB
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    import sys

    print(build(verbose=True, timeline="--timeline" in sys.argv[1:]))
