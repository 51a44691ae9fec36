"""The host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

Builds the packer, the quantiser, the C-ABI entry points (their argument checks; the kernel launchers
are stubbed) and the C oracle with -fsanitize=address,undefined into one executable
(tests/host/host_sanitize.cpp) and runs it: any memory error, leak or undefined operation fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2402_10517_amd", "csrc")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(os.path.join(ROCM, "include", "hip")),
                    reason="needs g++ and the HIP headers")
def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    objs = []
    for src in ("pack.cpp", "quantize.cpp", "api.cpp"):
        obj = str(tmp_path / (src + ".o"))
        subprocess.check_call(["g++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROCM, "include")] + SAN +
                              ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    obj = str(tmp_path / "oracle.o")
    subprocess.check_call(["gcc", "-std=c11", "-fopenmp"] + SAN + ["-c", os.path.join(ROOT, "oracle", "oracle.c"), "-o", obj])
    objs.append(obj)
    exe = str(tmp_path / "host_sanitize")
    subprocess.check_call(["g++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROCM, "include")] + SAN +
                          [os.path.join(ROOT, "tests", "host", "host_sanitize.cpp")] + objs +
                          ["-static-libasan", "-fopenmp", "-L" + os.path.join(ROCM, "lib"), "-lamdhip64",
                           "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-lpthread", "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "all checks held" in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
