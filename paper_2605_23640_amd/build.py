"""Builds libcacheprune.so (hand-written HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libcacheprune.so")
SOURCES = ["hash.hip", "table.hip", "verify.hip", "policy.hip", "annotate.hip", "spans.hip", "kv_move.hip"]
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
               # packed-FP32 instructions are kept out of all device code on the test machines
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force: bool = True) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    if not force and os.path.exists(LIB_PATH):
        newest = max(os.path.getmtime(os.path.join(CSRC, f)) for f in os.listdir(CSRC))
        if os.path.getmtime(LIB_PATH) >= newest:
            return LIB_PATH
    subprocess.run(["hipcc", *HIPCC_FLAGS, "-o", LIB_PATH, *srcs], check=True, cwd=CSRC)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
