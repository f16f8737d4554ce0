"""The oracle and the host-only part of the library under AddressSanitizer and UndefinedBehaviorSanitizer.

Two small programs (tests/sanitize/) are compiled from the same sources as the shared libraries, with
-fsanitize=address,undefined, and run once: a heap or stack overrun, a use after free, a signed overflow, a
misaligned or out-of-range access anywhere on the paths they walk ends the program with a report and a
non-zero status.  CPU only; the GPU side cannot be built with these sanitizers here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-g", "-O1", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    return r


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-std=c11", "-ffp-contract=off", *FLAGS, "-o", exe, os.path.join(SAN, "oracle_driver.c"),
         os.path.join(ROOT, "oracle", "pvq_oracle.c"), "-lm", "-lpthread"])
    r = run([exe], env=ENV, timeout=600)
    assert "oracle: ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"      # the library's headers use clang's vector types


@pytest.mark.skipif(not os.path.exists(CLANGXX) or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"),
                    reason="needs ROCm's clang++ and the HIP headers")
def test_host_side_of_the_library_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2410_16926_amd", "csrc")
    exe = str(tmp_path / "host_san")
    srcs = [os.path.join(SAN, "host_driver.cpp"), os.path.join(SAN, "kernel_stubs.cpp"),
            os.path.join(csrc, "pvq_host.cpp"), os.path.join(csrc, "pvq_fast8_tables.cpp")]
    run([CLANGXX, "-x", "c++", "-std=c++17", "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", *FLAGS, "-I/opt/rocm/include",
         f"-I{os.path.join(ROOT, 'include')}", f"-I{csrc}", "-o", exe, *srcs,
         "-x", "none", "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-lpthread"])
    r = run([exe], env=ENV, timeout=600)
    assert "host: ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
