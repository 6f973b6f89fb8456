"""AddressSanitizer + UndefinedBehaviorSanitizer over the native code that runs on the host: the C oracle and
the host-only logic of the C ABI.  CPU only; device code is not instrumented (the GPU sanitizer is not
available on the boxes this runs on), it is covered by the host's own bounds checks and the GPU parity tests."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1", "-static-libasan"]
# the sanitizer runtime is linked into the program; if something else is preloaded into the process it need not come first
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert res.returncode == 0, " ".join(cmd) + "\n" + res.stdout
    return res.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_c_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-std=c11", "-ffp-contract=off", *SAN, os.path.join(ROOT, "oracle", "gxpo_oracle.c"),
         os.path.join(ROOT, "tests", "san", "oracle_san.c"), "-o", exe, "-lm"])
    assert "oracle clean" in run([exe], env=ENV)


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"),
                    reason="needs g++ and the HIP headers")
def test_host_logic_of_the_c_abi_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
         "-I", os.path.join(ROOT, "paper_2605_06755_amd", "csrc"), os.path.join(ROOT, "paper_2605_06755_amd", "csrc", "gxpo_host.cpp"),
         os.path.join(ROOT, "tests", "san", "host_san.cpp"), "-o", exe, "-L", os.path.join(rocm, "lib"), "-lamdhip64",
         "-Wl,-rpath," + os.path.join(rocm, "lib")])
    # leak checking off here: the HIP runtime keeps process-lifetime allocations of its own
    out = run([exe], env=dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0")))
    assert "host logic clean" in out
