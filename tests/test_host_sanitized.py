"""The host side of the library -- argument checks, the closed-form plan, the launch geometry and
the workspace layout -- built with a plain C++ compiler under the address and undefined-behaviour
sanitizers (kernel launchers replaced by no-ops, <hip/hip_runtime.h> by a stand-in), and the CPU
boundary tests run against that build.  Device code is not covered: GPU sanitizers are not
available on the test machines."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_BUILD = os.path.join(ROOT, "tests", "host_build")
CSRC = os.path.join(ROOT, "paper_2605_06221_amd", "csrc")


def test_boundary_tests_pass_on_the_sanitized_host_build(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    lib = str(tmp_path / "libuniprefill_host_sanitized.so")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
           "-fno-sanitize-recover=undefined", "-x", "c++", "-I", HOST_BUILD, "-I", CSRC,
           os.path.join(CSRC, "up_api.hip"), os.path.join(HOST_BUILD, "launch_stubs.cpp"), "-o", lib]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    libasan = subprocess.run([gxx, "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    assert os.path.isabs(libasan) and os.path.exists(libasan), libasan
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is there stays
    env["LD_PRELOAD"] = libasan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"       # (the interpreter's own leaks are not the subject)
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    run = subprocess.run([sys.executable, os.path.join(HOST_BUILD, "run_boundary_tests.py"), lib], cwd=ROOT, env=env,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "passed" in run.stdout and "failed" not in run.stdout, run.stdout[-2000:]
    assert "AddressSanitizer" not in run.stdout and "runtime error:" not in run.stdout, run.stdout[-4000:]
