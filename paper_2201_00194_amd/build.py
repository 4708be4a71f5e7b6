"""Build the C-ABI library `libfamilyseer.so` for gfx950 with hipcc (in-tree)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfamilyseer.so")
CEILINGS = os.path.join(HERE, "fs_ceilings.bin")   # stand-alone microbenchmarks (csrc/fs_ceilings.hip)

SOURCES = ["fs_api.hip", "fs_model.hip", "fs_traverse_lds.hip", "fs_rank.hip", "fs_traverse_global.hip", "fs_segsum.hip", "fs_topk.hip", "fs_pack.hip", "fs_train.hip", "fs_gather.hip"]

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off",                     # sums must stay plain sequential adds
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-disable-promote-alloca-to-lds",   # the traversal kernel owns LDS from address 0
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           os.path.join(CSRC, "fs_ceilings.hip"), "-o", CEILINGS]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed (fs_ceilings):\n" +
                           "\n".join(l for l in res.stderr.splitlines() if noise not in l))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
