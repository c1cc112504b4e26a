"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

Builds (1) the C oracle and (2) the host part of the C ABI -- csrc/api.cpp: argument validation, work
planning, workspace carving -- with -fsanitize=address,undefined, the latter linked against launcher
stubs (tests/sanitize/launch_stubs.cpp) instead of the HIP kernels, then runs the oracle pins and the
ABI tests in a child process that has the sanitizer runtime preloaded.  Any report fails the test.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_LIB = os.path.join(ROOT, "tests", "sanitize", "libstructkv_hostsan.so")


def _build_host_library():
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    srcs = [os.path.join(ROOT, "paper_2604_06746_amd", "csrc", "api.cpp"),
            os.path.join(ROOT, "tests", "sanitize", "launch_stubs.cpp")]
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-fPIC",
           "-shared", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(rocm, "include")] + srcs + [
           "-o", HOST_LIB, "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.run(cmd, check=True)


@pytest.mark.skipif(os.environ.get("STRUCTKV_TEST_LIB") is not None, reason="already inside the sanitizer run")
def test_oracle_pins_and_abi_tests_under_asan_ubsan():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no libasan.so in this toolchain")
    _build_host_library()
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (env.get("LD_PRELOAD"), asan) if x)
    # python itself is not instrumented: no leak report at exit, and the runtime need not come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    env["STRUCTKV_ORACLE_SANITIZE"] = "1"
    env["STRUCTKV_TEST_LIB"] = HOST_LIB
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_abi.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in out
