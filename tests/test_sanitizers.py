"""The host-side code under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU oracle (oracle/fbq_oracle.c)
and the library's host part (csrc/fbq_api.cpp: descriptor checks, fbq_pack, argument validation) are compiled with
-fsanitize=address,undefined into one small program (tests/sanitize/san_driver.cpp) that runs pack / unpack /
quantize / reconstruct / linear on small layers and the entry points' error paths.  No GPU is involved: the
kernel launchers are stubs and nothing is ever launched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.exists(os.path.join(ROCM, "include", "hip", "hip_runtime.h")),
                    reason="needs g++ and the HIP runtime's headers")
def test_oracle_and_host_api_are_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    oracle_o = str(tmp_path / "fbq_oracle.o")
    subprocess.run(["gcc", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra", "-Wno-unknown-pragmas"] + san +
                   ["-c", os.path.join(ROOT, "oracle", "fbq_oracle.c"), "-o", oracle_o], check=True)
    exe = str(tmp_path / "san_driver")
    csrc = os.path.join(ROOT, "paper_2501_16385_amd", "csrc")
    # the library's host part is plain C++ against the HIP runtime's host API: g++ with the runtime's headers
    cmd = ["g++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROCM, "include")] + san + \
          ["-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "sanitize", "san_driver.cpp"), os.path.join(ROOT, "tests", "sanitize", "launch_stubs.cpp"),
           os.path.join(csrc, "fbq_api.cpp"), oracle_o, "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-lm", "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and "sanitize ok" in run.stdout, run.stdout[-3000:]
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout, run.stdout[-3000:]
