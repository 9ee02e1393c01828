"""The host layer of the library under AddressSanitizer + UndefinedBehaviorSanitizer on the CPU: csrc/api.hip and csrc/plan.hip are
compiled as plain C++ for the host, linked with stub launchers (tests/host/stub_kernels.cpp) and driven through the C ABI by
tests/host/abi_host_check.cpp.  No GPU code is built or run here; GPU sanitizers are not used."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_layer_is_clean_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    rocm = "/opt/rocm"
    if not gxx or not os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime.h")):
        pytest.skip("g++ or the HIP headers are not available")
    exe = str(tmp_path / "abi_host_check")
    # plain C++ build of the host layer: the HIP headers give the host API, the two device-side spellings that
    # api.hip uses for its built-in scratch array are given host meanings
    cmd = [gxx, "-x", "c++", "-std=c++17", "-O1", "-g", "-D__HIP_PLATFORM_AMD__",
           "-D__align__(n)=__attribute__((aligned(n)))", "-DHIP_SYMBOL(x)=(&x)",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-w",
           "-I", os.path.join(rocm, "include"), "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2506_15545_amd", "csrc"),
           os.path.join(ROOT, "paper_2506_15545_amd", "csrc", "api.hip"),
           os.path.join(ROOT, "paper_2506_15545_amd", "csrc", "plan.hip"),
           os.path.join(ROOT, "tests", "host", "stub_kernels.cpp"), os.path.join(ROOT, "tests", "host", "abi_host_check.cpp"),
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "ALL OK" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
