"""Builds libfreqcache.so (gfx950) in-tree with hipcc.  `python -m paper_2208_05321_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfreqcache.so")
SOURCES = ["fc_api.hip", "fc_prepare.hip", "fc_rows.hip", "fc_embedding.hip", "fc_sort.hip", "fc_worker.hip", "fc_gather.hip", "fc_freq.hip"]
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-fopenmp", "-pthread",
    "-ffp-contract=off",                                   # SGD step: rounded product, then subtract
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def build(verbose: bool = False, extra_flags=(), out: str | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra_flags, *[os.path.join(CSRC, s) for s in SOURCES], "-o", out or LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out or LIB


if __name__ == "__main__":
    print(build(verbose=True))
