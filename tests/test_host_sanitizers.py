"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code, run on the CPU (no GPU needed).

* the library's host side -- slab allocator and geometry (fs_pool), scheduler (fs_sched), the host validation and
  planning of the append and decode entry points -- compiled by hipcc with the host sanitizers on (device code
  is built as usual and never runs) and driven by tests/sanitize/fs_host_driver.cpp;
* the MFMA decode kernel's index arithmetic (the host + device functions of csrc/fs_attention.h), replayed item by
  item, tile by tile and lane by lane with every index asserted, by tests/sanitize/fs_index_check.cpp;
* the CPU oracle (oracle/fs_oracle.c), compiled by gcc with the sanitizers on and driven by
  tests/sanitize/oracle_driver.c.
A sanitizer report aborts the driver, a failed check makes it return 1; either fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUILD = os.path.join(ROOT, "_build")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    out = "\n".join(ln for ln in r.stdout.splitlines() if "packed-fp32-ops" not in ln)
    assert r.returncode == 0, f"{' '.join(cmd[:3])} ... failed ({r.returncode}):\n{out[-4000:]}"
    return out


def test_library_host_side_under_asan_and_ubsan():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    os.makedirs(BUILD, exist_ok=True)
    csrc = os.path.join(ROOT, "paper_2509_06261_amd", "csrc")
    srcs = [os.path.join(csrc, f) for f in ("fs_pool.hip", "fs_sched.hip", "fs_append.hip", "fs_attention.hip",
                                            "fs_attention_generic.hip", "fs_attention_mfma.hip")]
    exe = os.path.join(BUILD, "fs_host_driver")
    # -fno-gpu-sanitize: the sanitizers instrument the host pass only
    _run([hipcc, "--offload-arch=gfx950", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", *SAN, "-fno-gpu-sanitize", "-I", os.path.join(ROOT, "include"), "-I", csrc, *srcs,
          os.path.join(ROOT, "tests", "sanitize", "fs_host_driver.cpp"), "-o", exe])
    out = _run([exe], env=ENV, timeout=600)
    assert "fs_host_driver: 0 failed checks" in out, out[-2000:]


def test_decode_kernel_index_arithmetic_replayed_on_the_host():
    """tests/sanitize/fs_index_check.cpp: the MFMA decode kernel's own index functions, compiled for the host and run
    over every item, tile and lane of seeded launches with every table index and byte offset asserted."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    os.makedirs(BUILD, exist_ok=True)
    csrc = os.path.join(ROOT, "paper_2509_06261_amd", "csrc")
    srcs = [os.path.join(csrc, f) for f in ("fs_pool.hip", "fs_sched.hip", "fs_append.hip", "fs_attention.hip",
                                            "fs_attention_generic.hip", "fs_attention_mfma.hip")]
    exe = os.path.join(BUILD, "fs_index_check")
    _run([hipcc, "--offload-arch=gfx950", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", *SAN, "-fno-gpu-sanitize", "-I", os.path.join(ROOT, "include"), "-I", csrc, *srcs,
          "-x", "hip", os.path.join(ROOT, "tests", "sanitize", "fs_index_check.cpp"), "-o", exe])
    out = _run([exe], env=ENV, timeout=600)
    assert " 0 failed checks" in out and "fs_index_check:" in out, out[-2000:]
    print(out.strip().splitlines()[-1])


def test_oracle_under_asan_and_ubsan():
    if not shutil.which("gcc"):
        pytest.skip("gcc not found")
    os.makedirs(BUILD, exist_ok=True)
    exe = os.path.join(BUILD, "oracle_driver")
    _run(["gcc", "-std=c11", "-ffp-contract=off", "-pthread", "-Wall", *SAN,
          os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"])
    out = _run([exe], env=ENV, timeout=600)
    assert "oracle_driver: 0 failed checks" in out, out[-2000:]
