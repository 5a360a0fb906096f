"""The C ABI's host side (argument validation, the mapping of the six products onto the canonical
GEMM, the placement of the scratch areas inside the caller's workspace) built for the CPU with
AddressSanitizer and UndefinedBehaviorSanitizer and driven through every entry point.  The kernel
launchers are replaced by stubs that check the descriptions they receive; no GPU is involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
CSRC = os.path.join(ROOT, "paper_2401_11469_amd", "csrc")


def test_c_abi_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc in this environment")
    exe = str(tmp_path / "zr_host_check")
    cmd = [hipcc, "-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", "-g", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "zr_api.hip"), os.path.join(HERE, "stubs.cpp"), os.path.join(HERE, "driver.cpp"),
           "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout[-4000:]
    # (verify_asan_link_order=0: the environment may preload a library of its own ahead of the runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert run.stdout.strip().splitlines()[-1].startswith("OK"), run.stdout[-2000:]
