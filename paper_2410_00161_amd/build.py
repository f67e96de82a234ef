"""Builds libkvc.so (gfx950) from csrc/ with hipcc, in-tree.

    python -m paper_2410_00161_amd.build

hipcc cross-compiles without a GPU.  Objects go to _build/ (ignored by git); the
library lands next to this file so that it travels with the tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libkvc.so")

SOURCES = ["kvc_api.hip", "kvc_alloc.hip", "kvc_decode.hip", "kvc_evict.hip", "kvc_rank.hip", "kvc_window.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Per-source additions.  The decode kernels keep their matrix-core accumulators in ordinary
# vector registers: they are rescaled by plain multiplies whenever a running maximum moves, and
# in the accumulator file every such multiply costs a copy out and a copy back.
EXTRA_FLAGS = {"kvc_decode.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
               "kvc_window.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        raise RuntimeError("hipcc failed")
    return r


def build_library(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        _run([hipcc, *HIPCC_FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose:
            print(f"[kvc build] {src}", flush=True)

    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as ex:
        list(ex.map(one, zip(SOURCES, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC",
          "-o", LIB, *objs])
    if verbose:
        print(f"[kvc build] linked {LIB}", flush=True)
    return LIB


if __name__ == "__main__":
    build_library()
