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
LLVM_NM = shutil.which("nm") or "nm"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANGXX)), reason="ROCm compilers not found")
def test_abi_host_paths_are_clean_under_asan_and_ubsan(tmp_path):
    from concurrent.futures import ThreadPoolExecutor
    from paper_2511_18643_amd import build as kb
    chk = os.path.join(ROOT, "tests", "host_sanitize", "abi_host_check.cpp")
    chk_o, exe = (str(tmp_path / n) for n in ("abi_host_check.o", "abi_host_check"))
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]

    # host pass only, of every translation unit of the library (the host side and the per-variant launchers).  Each
    # unit refers to its device image by a symbol named after the unit's compilation id: the undefined
    # __hip_fatbin_* symbols are read back from the objects and given empty stand-ins.
    units = kb.translation_units()

    def host_only(unit):
        name, src, flags = unit
        obj = str(tmp_path / name)
        subprocess.run([HIPCC, "--cuda-host-only", "-c", "-O1", "-g", "-std=c++17", "-fPIC", *san,
                        "-Wno-unused-command-line-argument", *flags, src, "-o", obj], check=True, capture_output=True)
        return obj

    with ThreadPoolExecutor(max_workers=8) as pool:
        lib_objs = list(pool.map(host_only, units))
    nm = subprocess.run([LLVM_NM, "-u", *lib_objs], check=True, capture_output=True, text=True).stdout
    images = sorted({w for line in nm.splitlines() for w in line.split() if w.startswith("__hip_fatbin_")})
    assert len(images) == len(units), images
    stand_c, stand_o = str(tmp_path / "device_image_stand_ins.c"), str(tmp_path / "device_image_stand_ins.o")
    with open(stand_c, "w") as f:
        for sym in images:
            f.write('__attribute__((section(".hip_fatbin"), used)) unsigned long long %s[8] = {0};\n' % sym)
    subprocess.run([CLANGXX, "-x", "c", "-c", stand_c, "-o", stand_o], check=True, capture_output=True)
    lib_objs.append(stand_o)
    subprocess.run([CLANGXX, "-c", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", chk, "-o", chk_o], check=True, capture_output=True)
    subprocess.run([CLANGXX, "-fsanitize=address,undefined", *lib_objs, chk_o, "-L/opt/rocm/lib", "-lamdhip64",
                    "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("ok"), res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
