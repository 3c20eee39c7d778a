"""Host sanitizers (-fsanitize=address,undefined) on the CPU side: the oracle runs all its entry points on a small
graph inside one instrumented program, and the library's host code (api.hip: argument checks, context handling)
is rebuilt with the host pass instrumented and driven through its error paths by a native program.  No Python in
either process, so nothing is preloaded."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}"
    return r


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["g++", "-O1", "-g", "-std=c++17", *SAN, "-o", exe, os.path.join(ROOT, "oracle", "sanitize_main.cpp")])
    r = _run([exe], env=ENV, timeout=300)
    assert "oracle sanitizer run clean" in r.stdout and "ERROR" not in r.stderr and "runtime error" not in r.stderr


def test_abi_host_code_under_sanitizers(tmp_path):
    from paper_2305_16588_amd import build
    objs = []
    for src in build.SOURCES:
        obj = os.path.join(build.HERE, "_build", src.replace(".hip", ".o"))
        if src != "api.hip":
            objs.append(obj if os.path.exists(obj) else build._compile(src))
    api = str(tmp_path / "api_san.o")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    _run([build.HIPCC, *build.FLAGS, "-g", *host_san, "-c", os.path.join(build.CSRC, "api.hip"), "-o", api])
    lib = str(tmp_path / "liblegion_prep_san.so")
    _run([build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
          "-shared-libsan", "-o", lib, api, *objs])
    exe = str(tmp_path / "abi_san")
    clang = build.HIPCC.replace("hipcc", "amdclang++")
    runtime = _run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"]).stdout.strip()   # the shared sanitizer runtime
    _run([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan",
          "-I" + build.INCLUDE, os.path.join(ROOT, "tests", "abi_sanitize_main.cpp"), lib,
          "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib", "-Wl,-rpath," + os.path.dirname(runtime),
          "-o", exe])
    r = _run([exe], env=ENV, timeout=300)
    assert "abi sanitizer run clean" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
