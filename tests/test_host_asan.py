"""The library's host code (plan.cpp and the host halves of api.hip and executor.hip: validation, block generation,
CSR groupings, work lists and item cutting, workspace layout, copy lists, the executor) built for the CPU with
AddressSanitizer and UndefinedBehaviorSanitizer and driven through the C ABI by tests/host_asan/driver.cpp, with the GPU
side replaced by tests/host_asan/fake_device.cpp (device memory = host memory; every kernel launcher = a host walk over
the same arrays with the kernel's index arithmetic).  No GPU, no HIP runtime: g++ only."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_10620_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_asan")
BUILD = os.path.join(HERE, "_build")
FLAGS = ["-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_address_and_ub_sanitizers():
    os.makedirs(BUILD, exist_ok=True)
    srcs = [os.path.join(CSRC, f) for f in ("plan.cpp", "api.hip", "executor.hip")] + \
           [os.path.join(HERE, f) for f in ("fake_device.cpp", "driver.cpp")]

    def compile_one(src):
        obj = os.path.join(BUILD, os.path.basename(src) + ".o")
        r = subprocess.run(["g++", "-x", "c++"] + FLAGS + ["-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        return obj
    with ThreadPoolExecutor(max_workers=5) as ex:
        objs = list(ex.map(compile_one, srcs))
    exe = os.path.join(BUILD, "host_asan")
    r = subprocess.run(["g++", "-fsanitize=address,undefined"] + objs + ["-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, "150"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "host-asan ok" in r.stdout, (r.stdout[-3000:] + r.stderr[-6000:])
