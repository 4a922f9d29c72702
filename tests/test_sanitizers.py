"""The CPU oracle and the library's host-side validation layer under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU).

Each part is a small driver under ``tests/sanitize/`` that is compiled together with the code
under test with ``-fsanitize=address,undefined -fno-sanitize-recover=all`` and run as a program
of its own: any out-of-bounds access, use of freed memory, signed overflow, misaligned access or
bad shift ends it with a non-zero status and a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    res = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)
    assert res.returncode == 0, "sanitizer driver failed:\n%s\n%s" % (res.stdout[-2000:], res.stderr[-6000:])
    assert "ok" in res.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra", *SAN, "-static-libasan", "-static-libubsan",
                    os.path.join(ROOT, "oracle", "cube3d_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_san.c"),
                    "-o", exe], check=True)
    _run(exe)


HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/llvm/bin/clang++"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="ROCm compilers not found")
def test_c_abi_validation_layer_under_address_and_undefined_sanitizers(tmp_path):
    from paper_2105_14450_amd import build
    libdir = str(tmp_path / "lib")
    build.build_sanitized(libdir)
    exe = str(tmp_path / "abi_san")
    subprocess.run([CLANGXX, "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "sanitize", "abi_san.cpp"), "-L", libdir, "-lcube3d_san",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    _run(exe)
