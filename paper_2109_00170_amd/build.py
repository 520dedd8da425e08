"""Builds libalcs.so (HIP, gfx950) in-tree with hipcc.  Run as a script or call build()."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libalcs.so")
SOURCES = ["alcs_pack.cpp", "alcs_latency.cpp", "alcs_sparse.hip", "alcs_sparse_fused.hip", "alcs_sparse_dw.hip", "alcs_sparse_bf16.hip", "alcs_sparse_math16.hip", "alcs_depthwise.hip", "alcs_project.hip", "alcs_packdev.hip", "alcs_layoutdev.hip", "alcs_chanrec.hip", "alcs_dense.hip"]

# -packed-fp32-ops is switched off on purpose: packed fp32 VALU forms are not used.
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False) -> str:
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        # hipcc's host pass does not know the packed-fp32 feature; that warning is harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print("FAILED: %s\n%s" % (src, text), file=sys.stderr)
        elif verbose and text.strip():
            print(text)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


MEASURE_LIB = os.path.join(HERE, "libalcs_measure.so")


def build_measure(verbose: bool = False) -> str:
    """The measurement build: the same library with -DALCS_MEASURE=1, in which the option
    ``measure_skip`` makes the kernels of alcs_sparse_conv skip phases (staging, multiply, stores)
    so that the others can be timed.  Never loaded by the package (point ALCS_LIBRARY at it for a
    measurement run); needs the objects of build() to exist."""
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        if src in ("alcs_pack.cpp", "alcs_sparse.hip"):
            obj = os.path.join(CSRC, os.path.splitext(src)[0] + "_measure.o")
            cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj, "-DALCS_MEASURE=1"] + FLAGS
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL if not verbose else None,
                           stderr=subprocess.DEVNULL if not verbose else None)
        objs.append(obj)
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", MEASURE_LIB] + objs)
    return MEASURE_LIB


if __name__ == "__main__":
    print(build(verbose=True))
    if "--measure" in sys.argv:
        print(build_measure(verbose=True))
