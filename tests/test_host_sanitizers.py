"""AddressSanitizer + UndefinedBehaviorSanitizer run of the library's host code (argument validation, shape
checks, workspace arithmetic): tests/host_checks.c, a plain-C client of include/moespec.h, is linked against a
build of the library whose host side is instrumented, and must finish without a sanitizer report.  No GPU is
needed: every call in it is answered before any device work."""
import os
import shutil
import subprocess

import pytest

from paper_2602_16052_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _clang():
    for cand in ("/opt/rocm/llvm/bin/clang", shutil.which("amdclang"), shutil.which("clang")):
        if cand and os.path.exists(cand):
            return cand
    return None


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    clang = _clang()
    if clang is None:
        pytest.skip("no clang to build the instrumented client with")
    lib = build.build_host_sanitizer_library(str(tmp_path))
    exe = str(tmp_path / "host_checks")
    cc = subprocess.run([clang, "-std=c11", "-O1", "-g", "-Wall", "-Wextra", "-pedantic", "-Werror",
                         "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                         "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host_checks.c"),
                         lib, "-Wl,-rpath," + str(tmp_path), "-o", exe],
                        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert cc.returncode == 0, cc.stdout
    env = dict(os.environ)
    # the HIP runtime that the library links keeps allocations until exit: leak detection is not the point here
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout
    assert "host checks passed" in run.stdout
    assert "AddressSanitizer" not in run.stdout and "runtime error" not in run.stdout, run.stdout
