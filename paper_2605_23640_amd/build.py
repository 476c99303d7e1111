"""Builds libcacheprune.so (hand-written HIP, gfx950 only) in-tree with hipcc.

Every source is compiled on its own (in parallel) with warnings as errors, the
device assembly of each is checked for packed-FP32 arithmetic, then the objects
are linked.  Intermediate files go to ``_build/`` beside this file.
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libcacheprune.so")
SOURCES = ["hash.hip", "table.hip", "verify.hip", "policy.hip", "annotate.hip", "spans.hip", "kv_move.hip"]
# Packed FP32 arithmetic (v_pk_add/mul/fma_f32) is kept out of all device code on the test machines:
# the target feature is switched off for the compiler.  -Xclang options reach the host compilation
# too, where the feature does not exist; the host pass says so in one fixed line, which is the only
# compiler output that is let through.
NO_PACKED_FP32 = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Werror", *NO_PACKED_FP32]
PACKED_FP32 = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")


def compile_hip(src: str, obj_dir: str, flags=HIPCC_FLAGS) -> str:
    """hipcc -c one source into obj_dir; raises on any compiler message besides the host pass's note
    about the device-only feature, and if the device assembly holds a packed-FP32 instruction."""
    stem = os.path.splitext(os.path.basename(src))[0]
    obj = os.path.join(obj_dir, stem + ".o")
    p = subprocess.run(["hipcc", *flags, "-save-temps=obj", "-c", "-o", obj, src], cwd=os.path.dirname(src),
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    said = [ln for ln in p.stdout.splitlines() if ln.strip() and ln.strip() != HOST_PASS_NOTE]
    if p.returncode != 0 or said:
        raise RuntimeError(f"hipcc {os.path.basename(src)} (exit {p.returncode}):\n" + "\n".join(said))
    asm = os.path.join(obj_dir, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")
    with open(asm) as f:
        hits = [ln.strip() for ln in f if PACKED_FP32.search(ln)]
    if hits:
        raise RuntimeError(f"{os.path.basename(src)}: packed-FP32 instructions in the device code: {hits[:3]}")
    return obj


def build(force: bool = True) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    if not force and os.path.exists(LIB_PATH):
        newest = max(os.path.getmtime(os.path.join(CSRC, f)) for f in os.listdir(CSRC))
        if os.path.getmtime(LIB_PATH) >= newest:
            return LIB_PATH
    shutil.rmtree(OBJ_DIR, ignore_errors=True)
    os.makedirs(OBJ_DIR)
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s: compile_hip(s, OBJ_DIR), srcs))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs], check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
