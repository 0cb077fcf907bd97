"""Build libsapo.so (HIP, gfx950 only) in-tree next to this file.

    python -m paper_2509_08721_amd.build

hipcc cross-compiles for gfx950 without a GPU.  Objects are compiled in parallel and
linked into one shared library; nothing is installed outside the source tree.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsapo.so")

SOURCES = ["api.hip", "kernels_generic.hip", "kernels_mfma.hip", "kernels_decode.hip", "decode_persist.hip", "train.hip"]
# SAPO_PERSIST_TRACE=1 in the environment: diagnostic build of the persistent decode kernel (per-phase tick counters)
FLAGS = (["-DSAPO_PERSIST_TRACE"] if os.environ.get("SAPO_PERSIST_TRACE") == "1" else []) + ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the first kernel arguments arrive in scalar registers with the wave instead of through a load
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-function", "-Wno-unused-variable"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build_library(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    hipcc = _hipcc()
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    objs = [os.path.join(BUILD, s.replace(".hip", ".o")) for s in srcs]
    cmds = [[hipcc] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(srcs, objs)]
    with cf.ThreadPoolExecutor(max_workers=min(8, len(cmds))) as ex:
        for s, out in zip(srcs, ex.map(_run, cmds)):
            if verbose and out.strip():
                print("[%s]\n%s" % (s, out))
    _run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
