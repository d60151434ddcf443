"""The host side of the HIP library (argument validation, launch planning, the Option II formula)
under AddressSanitizer and UBSan.  GPU sanitizers are not available, so only host code is
instrumented (hipcc: each -fsanitize= directly after -Xarch_host); a C client built with the same
compiler sweeps sizes through the planner and calls the validators with host arrays."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = "/opt/rocm/bin/hipcc"
CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.timeout(600)
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    if not (os.path.exists(HIPCC) and os.path.exists(CLANG)):
        pytest.skip("needs the ROCm compilers")
    if not glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"):
        pytest.skip("the ROCm clang has no host AddressSanitizer runtime")
    lib = str(tmp_path / "libcore_hip_san.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-shared", "-fPIC",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=undefined", "-Wno-unknown-warning-option",
                    "-o", lib, os.path.join(ROOT, "paper_2309_13307_amd", "csrc", "core_api.hip")],
                   check=True, capture_output=True, text=True)
    exe = str(tmp_path / "abi_san_client")
    subprocess.run([CLANG, "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-g",
                    "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "native", "abi_san_client.c"),
                    "-o", exe, "-L", str(tmp_path), "-l:libcore_hip_san.so",
                    f"-Wl,-rpath,{tmp_path}", "-Wl,-rpath,/opt/rocm/lib"], check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert res.returncode == 0, (res.returncode, res.stdout[-2000:], res.stderr[-4000:])
    assert "sanitized client ok" in res.stdout
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr
