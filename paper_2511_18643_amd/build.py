"""Builds libkitty.so (hipcc, gfx950) next to this file.  Run as `python -m paper_2511_18643_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libkitty.so")
SRC = os.path.join(HERE, "csrc", "kitty_api.hip")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",      # register / scratch report per kernel, checked below
]


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *(extra or []), SRC, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building libkitty.so")
    usage = kernel_resource_usage(res.stderr)
    # The decode kernel updates its running sums with an in-place FMA written as inline code, whose operands must
    # live in registers: a variant that spills to scratch memory is a build error, not a slow kernel.
    spilled = {k: v for k, v in usage.items() if v.get("ScratchSize [bytes/lane]", 0) > 0}
    if spilled:
        raise RuntimeError("kernels spill registers to scratch memory: %s" % sorted(spilled))
    if verbose:
        noise = ("is not a recognized feature for this target", "warnings generated")
        sys.stderr.write("".join(l + "\n" for l in res.stderr.splitlines()
                                 if ("warning:" in l or "error:" in l) and not any(n in l for n in noise)))
        worst = max(usage.items(), key=lambda kv: kv[1].get("VGPRs", 0), default=None)
        if worst:
            print("%d kernels, none uses scratch memory; most registers: %d VGPRs" % (len(usage), worst[1]["VGPRs"]), flush=True)
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
