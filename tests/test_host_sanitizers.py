"""The argument checks of every C-ABI entry point, once more, with the library's HOST code built under
AddressSanitizer and UndefinedBehaviorSanitizer (device code is compiled as usual; sanitizers for GPU
code are not used).  A C driver (tests/host_abi_san.c) links against that build and calls the same error
paths as test_host_abi.py; nothing it calls reaches a launch, so it runs without a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="needs the ROCm clang")
def test_argument_checks_under_host_sanitizers(tmp_path):
    from paper_2603_06619_amd import build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    lib = build.build(extra_flags=san, lib_path=str(tmp_path / "libnat_hip_san.so"), obj_dir=str(tmp_path / "obj"),
                      link_flags=["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"])
    exe = str(tmp_path / "host_abi_san")
    cmd = [CLANG, "-std=c11", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host_abi_san.c"), lib, "-Wl,-rpath," + str(tmp_path), "-lm", "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0 and "host_abi_san OK" in run.stdout, run.stdout[-4000:]
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout, run.stdout[-4000:]
    shutil.rmtree(tmp_path / "obj", ignore_errors=True)
