"""Builds libmoespec.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libmoespec.so")
SOURCES = ("api.hip", "route.hip", "budget.hip", "prologue.hip", "expert_ffn.hip", "analysis.hip", "stack.hip")

# Packed-FP32 instructions are disabled for all device code (hipcc's host pass warns that it does
# not know the feature; that warning is harmless).
HIPCC_FLAGS = ("--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument")


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found (set HIPCC or add /opt/rocm/bin to PATH)")


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source into paper_2602_16052_amd/libmoespec.so; returns its path."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH + ".tmp"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    if verbose and out.strip():
        print(out, file=sys.stderr)
    return LIB_PATH


def build_host_sanitizer_library(out_dir: str) -> str:
    """The library with AddressSanitizer and UndefinedBehaviorSanitizer instrumentation in its HOST code only
    (GPU sanitizers are not used); the device code is compiled unoptimised to keep the build short.  For the
    host-side checks in tests/; never loaded by the product path.  Returns the path of the library."""
    out = os.path.join(out_dir, "libmoespec_hostsan.so")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"]
    cmd = [hipcc_path(), *flags, "-Xarch_device", "-O0", "-Xarch_host", "-O1",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in res.stdout.splitlines()
                                                          if "packed-fp32-ops" not in l))
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
