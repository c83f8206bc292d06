"""Builds libkitty.so (hipcc, gfx950) next to this file: the host side and one translation unit per record variant,
compiled side by side, then linked.  Run as `python -m paper_2511_18643_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libkitty.so")
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",      # register / scratch report per kernel, checked below
]

# record variants (16-channel boost blocks, 4-bit Values): one translation unit each (csrc/kitty_variant.hip), the
# same set kitty_api.hip dispatches to
VARIANTS = [(nb, 0) for nb in range(9)] + [(nb, 1) for nb in range(9)]


def translation_units(extra: list[str] | None = None) -> list[tuple[str, str, list[str]]]:
    """(object name, source, flags) of every translation unit of the library."""
    extra = list(extra or [])
    units = [("kitty_api.o", os.path.join(CSRC, "kitty_api.hip"), extra)]
    for nb, v4 in VARIANTS:
        units.append((f"kitty_variant_nb{nb}_v{4 if v4 else 2}.o", os.path.join(CSRC, "kitty_variant.hip"),
                      extra + [f"-DKITTY_VARIANT_NB={nb}", f"-DKITTY_VARIANT_V4={v4}"]))
    return units


def build(verbose: bool = False, extra: list[str] | None = None, jobs: int | None = None) -> str:
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    units = translation_units(extra)
    jobs = jobs or max(1, min(len(units), os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "16"))))

    def compile_one(unit):
        name, src, flags = unit
        obj = os.path.join(OBJ_DIR, name)
        cmd = [hipcc, *FLAGS, *flags, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        return obj, subprocess.run(cmd, capture_output=True, text=True)

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(compile_one, units))
    remarks = ""
    for obj, res in results:
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError("hipcc failed compiling %s" % os.path.basename(obj))
        remarks += res.stderr
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for o, _ in results], "-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed linking libkitty.so")
    usage = kernel_resource_usage(remarks)
    # The decode kernel updates its running sums with an in-place FMA written as inline code, whose operands must
    # live in registers: a variant that spills to scratch memory is a build error, not a slow kernel.
    spilled = {k: v for k, v in usage.items() if v.get("ScratchSize [bytes/lane]", 0) > 0}
    if spilled:
        raise RuntimeError("kernels spill registers to scratch memory: %s" % sorted(spilled))
    if verbose:
        noise = ("is not a recognized feature for this target", "warnings generated")
        sys.stderr.write("".join(l + "\n" for l in remarks.splitlines()
                                 if ("warning:" in l or "error:" in l) and not any(n in l for n in noise)))
        worst = max(usage.items(), key=lambda kv: kv[1].get("VGPRs", 0), default=None)
        if worst:
            print("%d kernels in %d translation units, none uses scratch memory; most registers: %d VGPRs"
                  % (len(usage), len(units), worst[1]["VGPRs"]), flush=True)
    return LIB


def kernel_resource_usage(remarks: str) -> dict[str, dict[str, int]]:
    """Parses hipcc's -Rpass-analysis=kernel-resource-usage remarks: {mangled kernel name: {field: value}}."""
    import re
    out: dict[str, dict[str, int]] = {}
    cur = None
    for line in remarks.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return out


if __name__ == "__main__":
    print(build(verbose=True))
