"""Compile the native pieces in-tree.

Three independent shared objects are produced:

* ``paper_2307_05740_amd/libarrow.so``        -- HIP kernels + host decomposition + C-ABI (hipcc, gfx950)
* ``paper_2307_05740_amd/synth/libsynth.so``  -- seeded input generators (gcc)
* ``oracle/liboracle.so``                     -- the fp64 CPU checker (gcc); building it is not using it

``python -m paper_2307_05740_amd._build arrow --sanitize`` builds ``arrow_host_check_asan``
instead: the host half of the library (everything but the kernels) as a CPU-only program under
AddressSanitizer and UndefinedBehaviorSanitizer; ``tests/test_host_sanitizer.py`` runs it.

Nothing here is run at import time; ``__graft_entry__.build()`` and the
``python -m paper_2307_05740_amd._build`` command line call it.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
REPO_DIR = os.path.dirname(PKG_DIR)

ARROW_LIB = os.path.join(PKG_DIR, "libarrow.so")
SYNTH_LIB = os.path.join(PKG_DIR, "synth", "libsynth.so")
ORACLE_LIB = os.path.join(REPO_DIR, "oracle", "liboracle.so")

HIP_SOURCES = ["csrc/decompose.cpp", "csrc/layout.cpp", "csrc/abi.cpp", "csrc/kernels.hip",
               "csrc/csf3.cpp", "csrc/mttkrp.hip", "csrc/probe.hip", "csrc/static_scratch.hip"]


def _run(cmd: list[str]) -> None:
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout)
        raise RuntimeError("build step failed: " + " ".join(cmd))
    # keep real diagnostics, drop the host pass's note about the device-only feature flag
    for line in proc.stdout.splitlines():
        if "packed-fp32-ops" in line and "not a recognized feature" in line:
            continue
        if line.strip():
            sys.stderr.write(line + "\n")


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_synth() -> str:
    src = os.path.join(PKG_DIR, "synth", "synth.c")
    _run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
          "-o", SYNTH_LIB, src, "-lm"])
    return SYNTH_LIB


def build_oracle() -> str:
    srcs = [os.path.join(REPO_DIR, "oracle", f) for f in ("spmm_oracle.c", "mttkrp_oracle.c")]
    _run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
          "-ffp-contract=off", "-o", ORACLE_LIB] + srcs + ["-lm"])
    return ORACLE_LIB


def build_arrow() -> str:
    srcs = [os.path.join(PKG_DIR, s) for s in HIP_SOURCES]
    cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-fopenmp", "-Wall", "-Wno-unused-result",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(REPO_DIR, "include"), "-x", "hip"]
    cmd += srcs + ["-o", ARROW_LIB]
    _run(cmd)
    return ARROW_LIB


HOST_CHECK = os.path.join(PKG_DIR, "arrow_host_check")
HOST_SOURCES = ["csrc/decompose.cpp", "csrc/layout.cpp", "csrc/abi.cpp", "csrc/csf3.cpp", "csrc/host_check.cpp"]


def build_host_check(sanitize: bool = True) -> str:
    """CPU-only program that runs the host half of the library (CSR validation, decomposition,
    packing, self-check, export, save / load / repack, the fibre builder) with the kernel
    launchers stubbed out; with ``sanitize`` it is built with AddressSanitizer and
    UndefinedBehaviorSanitizer, every report fatal.  g++ compiles the same sources hipcc does."""
    srcs = [os.path.join(PKG_DIR, s) for s in HOST_SOURCES]
    rocm_inc = os.path.join(os.path.dirname(os.path.dirname(_hipcc())), "include")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fopenmp", "-Wall", "-Wno-unused-result", "-Wno-unknown-pragmas",
           "-D__HIP_PLATFORM_AMD__", "-I", rocm_inc, "-I", os.path.join(REPO_DIR, "include")]
    if sanitize:
        cmd += ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    out = HOST_CHECK + ("_asan" if sanitize else "")
    _run(cmd + srcs + ["-o", out])
    return out


def build_all() -> None:
    build_synth()
    build_oracle()
    build_arrow()


if __name__ == "__main__":
    what = sys.argv[1:] or ["all"]
    for w in what:
        if w == "--sanitize":
            continue
        if w == "arrow" and "--sanitize" in what:
            build_host_check(sanitize=True)        # the host half of the library under ASan + UBSan
            continue
        {"all": build_all, "synth": build_synth, "oracle": build_oracle, "arrow": build_arrow,
         "host_check": lambda: build_host_check(sanitize=False)}[w]()
    print("built:", ", ".join(what))
