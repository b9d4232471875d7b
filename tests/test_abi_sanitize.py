"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer: build.py --sanitize builds a
second library with instrumented host code, and a small C program (tests/host/abi_sanitize_driver.c) walks
through the argument checks of every entry point against it.  No GPU is needed: every call stops at a host
check.  The sanitizers must stay silent and the program must print "ok"."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG) or shutil.which("hipcc") is None, reason="needs ROCm's clang and hipcc")
def test_host_side_of_the_boundary_under_sanitizers():
    from paper_1805_08899_amd import build
    lib = build.build_library(sanitize=True, verbose=False)
    syms = subprocess.run(["nm", "-D", lib], capture_output=True, text=True).stdout
    assert "__asan_" in syms and "__ubsan_" in syms, "the host code is not instrumented"
    libdir = os.path.dirname(lib)
    exe = os.path.join(libdir, "abi_sanitize_driver")
    rt_dir = os.path.dirname(subprocess.run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"],
                                            capture_output=True, text=True).stdout.strip())
    cmd = [CLANG, "-std=c99", "-g", "-Wall", "-Werror", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-shared-libsan", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host", "abi_sanitize_driver.c"), "-o", exe, "-L", libdir, "-lechoattn_san",
           f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{rt_dir}"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout, r.stderr)
    assert r.stdout.strip().endswith("ok"), r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
