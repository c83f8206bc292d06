"""The host side of libkitty (argument validation, split planning, the dispatch around the launches) built without
its device code under AddressSanitizer and UndefinedBehaviorSanitizer, and driven by tests/host_sanitize/
abi_host_check.cpp with the same kind of calls as test_abi_host.py: invalid arguments, plan sweeps, extreme
sizes.  Nothing is launched, so no GPU is needed; any sanitizer report makes the program exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="ROCm compilers not found")
def test_abi_host_paths_are_clean_under_asan_and_ubsan(tmp_path):
    api = os.path.join(ROOT, "paper_2511_18643_amd", "csrc", "kitty_api.hip")
    chk = os.path.join(ROOT, "tests", "host_sanitize", "abi_host_check.cpp")
    lib_o, chk_o, exe = (str(tmp_path / n) for n in ("kitty_api_host.o", "abi_host_check.o", "abi_host_check"))
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    # host pass only; -fuse-cuid=none gives the reference to the device image the fixed name the check program defines
    subprocess.run([HIPCC, "--cuda-host-only", "-fuse-cuid=none", "-c", "-O1", "-g", "-std=c++17", "-fPIC", *san,
                    "-Wno-unused-command-line-argument", api, "-o", lib_o], check=True, capture_output=True)
    subprocess.run([CLANGXX, "-c", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", chk, "-o", chk_o], check=True, capture_output=True)
    subprocess.run([CLANGXX, "-fsanitize=address,undefined", lib_o, chk_o, "-L/opt/rocm/lib", "-lamdhip64",
                    "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("ok"), res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
