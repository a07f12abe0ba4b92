"""The library's host code (argument checks, shape bookkeeping, the Eq. 3 schedule: everything in
csrc/stem_api.cpp) built for the CPU only with AddressSanitizer and UndefinedBehaviorSanitizer, the
kernel launchers replaced by no-op stand-ins (tests/host_launch_stubs.cpp), and the host ABI tests run
against that build in a child process.  Any out-of-bounds access, overflow or misaligned access in
the host code aborts the child."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_06274_amd", "csrc")


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(shutil.which("g++") is None or _runtime("libasan.so") is None or _runtime("libubsan.so") is None
                    or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"),
                    reason="needs g++ with the ASan/UBSan runtimes and the HIP headers")
def test_host_abi_under_address_and_ub_sanitizers(tmp_path):
    lib = str(tmp_path / "libstem_host_san.so")
    build = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-fno-omit-frame-pointer",
             "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
             os.path.join(CSRC, "stem_api.cpp"), os.path.join(ROOT, "tests", "host_launch_stubs.cpp"), "-o", lib]
    res = subprocess.run(build, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    preload = [_runtime("libasan.so"), _runtime("libubsan.so")]
    if os.environ.get("LD_PRELOAD"):
        preload.append(os.environ["LD_PRELOAD"])
    env = dict(os.environ, LD_PRELOAD=":".join(preload), STEM_HIP_LIBRARY=lib,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               PYTHONDONTWRITEBYTECODE="1")
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_host_abi.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-3000:])
    assert "passed" in run.stdout and "Sanitizer" not in run.stderr and "runtime error" not in run.stderr
