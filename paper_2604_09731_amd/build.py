"""Builds the C-ABI library (libsmart_tree.so) in-tree with hipcc for gfx950, and beside it the timeline build
(libsmart_tree_timeline.so: the same library with wall-clock stamps in the attention kernels, for
`python -m paper_2604_09731_amd.timeline`; nothing else loads it)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libsmart_tree.so")
TIMELINE_LIB = os.path.join(HERE, "libsmart_tree_timeline.so")
TIMELINE_SOURCE = "tva_mfma.hip"        # the one source with stamps (-DSMART_TVA_TIMELINE)
OBJ_DIR = os.path.join(HERE, "_build")

HIP_SOURCES = ["smart_ctx.hip", "tree_pack_accept.hip", "kv_cache_write.hip", "tva_general.hip",
               "tva_mfma.hip", "tva_api.hip", "tva_static.hip", "smart_select_device.hip", "tree_rope.hip",
               "tree_accept_sample.hip"]
HOST_SOURCES = ["smart_select.cpp", "smart_cost_model.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
             # the compiler must not form packed fp32 instructions on this target
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-function"]
# selection decisions must be bit-identical everywhere: no FMA contraction
HIP_EXTRA = {"smart_select_device.hip": ["-ffp-contract=off"]}
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-ffp-contract=off", "-I", INCLUDE, "-Wall", "-pthread"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("build step failed: " + " ".join(cmd))
    if out.strip():
        print(out)


def build_library(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = []
    for s in HIP_SOURCES:
        o = os.path.join(OBJ_DIR, s + ".o")
        _run([HIPCC, *HIP_FLAGS, *HIP_EXTRA.get(s, []), "-c", os.path.join(CSRC, s), "-o", o])
        objs.append(o)
    for s in HOST_SOURCES:
        o = os.path.join(OBJ_DIR, s + ".o")
        _run(["g++", *HOST_FLAGS, "-c", os.path.join(CSRC, s), "-o", o])
        objs.append(o)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-pthread"])
    if verbose:
        print("built", LIB)
    # the timeline build: one object compiled again with the stamps, the rest shared
    plain = os.path.join(OBJ_DIR, TIMELINE_SOURCE + ".o")
    stamped = os.path.join(OBJ_DIR, TIMELINE_SOURCE + ".timeline.o")
    _run([HIPCC, *HIP_FLAGS, "-DSMART_TVA_TIMELINE", "-c", os.path.join(CSRC, TIMELINE_SOURCE), "-o", stamped])
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", TIMELINE_LIB,
          *[stamped if o == plain else o for o in objs], "-pthread"])
    if verbose:
        print("built", TIMELINE_LIB)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
