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
    if verbose:
        noise = "is not a recognized feature for this target"
        sys.stderr.write("".join(l + "\n" for l in res.stderr.splitlines() if noise not in l and "warnings generated" not in l))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
