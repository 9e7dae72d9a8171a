"""Builds liboptireduce_hip.so for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2310_06993_amd.build [--microbench]

Every translation unit is compiled on every call of build(); the block-size classes compile in
parallel.  Objects go to _build/ (not tracked); the library lands next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "liboptireduce_hip.so")
CLASSES = (0, 11, 12, 13, 14, 15, 16)

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
FLAGS += os.environ.get("OR_HIPCC_EXTRA", "").split()   # e.g. -DOR_SWAP_STAGES=1 when trying a variant


def _compile(job):
    src, obj, extra = job
    cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("hipcc failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    return obj


def build(jobs: int | None = None) -> str:
    os.makedirs(OBJ, exist_ok=True)
    work = [(os.path.join(CSRC, "optireduce_api.hip"), os.path.join(OBJ, "api.o"), [])]
    for c in CLASSES:
        work.append((os.path.join(CSRC, "inst.hip"), os.path.join(OBJ, "inst_%d.o" % c), ["-DOR_K=%d" % c]))
    jobs = jobs or min(8, os.cpu_count() or 1, len(work))
    with ThreadPoolExecutor(jobs) as ex:
        objs = list(ex.map(_compile, work))
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", tmp]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    os.replace(tmp, LIB)
    return LIB


MICROBENCH_SRC = os.path.join(PKG, "microbench", "or_microbench.hip")
MICROBENCH = os.path.join(PKG, "microbench", "or_microbench")


def build_microbench() -> str:
    """The standalone measurement program behind the design notes (not loaded by the library or the tests)."""
    cmd = [HIPCC, *[f for f in FLAGS if f not in ("-fPIC", "-fno-gpu-rdc")], MICROBENCH_SRC, "-o", MICROBENCH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("hipcc failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    return MICROBENCH


if __name__ == "__main__":
    print(build())
    if "--microbench" in sys.argv:
        print(build_microbench())
