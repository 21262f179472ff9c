"""Builds libgto.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgto.so")
SOURCES = ["gto_api.hip", "gto_rows.hip", "gto_tree.hip", "gto_fused.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-fno-honor-nans", "-Wall", "-Wno-unused-command-line-argument",
]


def build_lib(verbose: bool = False, extra=(), out: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra, *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    # hipcc's host pass prints one line per file about the device-only target feature: harmless
    res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err, flush=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed with status {res.returncode}")
    return out


if __name__ == "__main__":
    print(build_lib(verbose=True))
